// Inter-layer attention similarity for the offline layer grouping (the paper's "Attention Similarity
// Measurement"): for head h and layers a, b, the Jensen-Shannon divergence of the two layers' attention
// rows, averaged over the sampled rows; the similarity is 1 minus that average with base-2 logarithms
// (base-2 JS lies in [0, 1], so identical rows give 1 and rows with disjoint support give 0).
//
// Elementwise work followed by a reduction.  A workgroup takes one head and a block pair (A, B) of kBL layers each
// (A <= B) and walks the heads' rows once, 16 bytes per lane and load: every element of up to 2 kBL layers is loaded
// once, its logarithm taken once, and all the kBL x kBL (or, on the diagonal, kBL (kBL - 1) / 2) layer pairs of the
// block pair are accumulated from those registers.  Against one workgroup per layer pair this reads each row
// ceil(L / kBL) times instead of L - 1 times (32 layers: 4 instead of 31) and takes 1 + 2 / kBL instead of 3
// logarithms per pair and element.  Nothing here is on the inference path; it feeds pod_group_layers.
#include "pod_internal.h"

namespace {

constexpr int kSimThreads = 256;
constexpr int kBL = 8;   // layers per block
typedef __attribute__((ext_vector_type(4))) float sim_f4;

// (subnormal probabilities count as 0: the hardware logarithm flushes them, and x log x < 1e-35 there)
constexpr float kMinNormal = 1.17549435e-38f;

// sum over the 4 elements of p log2(p / m) + q log2(q / m) with m = (p + q) / 2 and 0 log 0 = 0; lp, lq = log2 of p, q
__device__ inline float js_term4(const sim_f4 &p, const sim_f4 &lp, const sim_f4 &q, const sim_f4 &lq)
{
    float t = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float lm = __log2f(0.5f * (p[e] + q[e]));
        if (p[e] >= kMinNormal) t += p[e] * (lp[e] - lm);
        if (q[e] >= kMinNormal) t += q[e] * (lq[e] - lm);
    }
    return t;
}

// att: [L][H][R][n] probabilities (rows sum to 1); sim: [H][L][L]
__global__ __launch_bounds__(kSimThreads) void similarity_kernel(const float *__restrict__ att, int L, int H, int R, int n,
                                                                 float *__restrict__ sim)
{
    // block pair index -> (A, B), A <= B
    const int nblk = (L + kBL - 1) / kBL;
    int A = 0, rem = blockIdx.x;
    while (rem >= nblk - A) { rem -= nblk - A; ++A; }
    const int B = A + rem, h = blockIdx.y;
    const bool diag = A == B;
    const size_t rows = (size_t)R * n; // the R rows of one (layer, head) are contiguous
    const size_t vec = rows / 4;       // (the entry point takes R * n in multiples of 4 only)
    float acc[kBL][kBL];
#pragma unroll
    for (int i = 0; i < kBL; ++i)
#pragma unroll
        for (int j = 0; j < kBL; ++j) acc[i][j] = 0.f;
    auto row_ptr = [&](int layer) { return att + ((size_t)(layer < L ? layer : L - 1) * H + h) * rows; };
    auto log4 = [](const sim_f4 &x) {
        sim_f4 l;
#pragma unroll
        for (int e = 0; e < 4; ++e) l[e] = __log2f(x[e]);
        return l;
    };
    auto accumulate = [&](const sim_f4 (&xa)[kBL], const sim_f4 (&la)[kBL], const sim_f4 (&xb)[kBL], const sim_f4 (&lb)[kBL]) {
#pragma unroll
        for (int i = 0; i < kBL; ++i)
#pragma unroll
            for (int j = 0; j < kBL; ++j)
                if (!diag || i < j) acc[i][j] += js_term4(xa[i], la[i], xb[j], lb[j]);   // (wave-uniform)
    };
    for (size_t v = threadIdx.x; v < vec; v += kSimThreads) {
        sim_f4 xa[kBL], la[kBL], xb[kBL], lb[kBL];
#pragma unroll
        for (int i = 0; i < kBL; ++i) xa[i] = ((const sim_f4 *)row_ptr(A * kBL + i))[v];
        if (!diag) {
#pragma unroll
            for (int j = 0; j < kBL; ++j) xb[j] = ((const sim_f4 *)row_ptr(B * kBL + j))[v];
        }
#pragma unroll
        for (int i = 0; i < kBL; ++i) la[i] = log4(xa[i]);
        if (!diag) {
#pragma unroll
            for (int j = 0; j < kBL; ++j) lb[j] = log4(xb[j]);
            accumulate(xa, la, xb, lb);
        } else {
            accumulate(xa, la, xa, la);
        }
    }
    // workgroup reduction, pair by pair
    __shared__ float part[kSimThreads / 64][kBL * kBL];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < kBL; ++i)
#pragma unroll
        for (int j = 0; j < kBL; ++j) {
            float t = acc[i][j];
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) t += __shfl_xor(t, off);
            if (lane == 0) part[wave][i * kBL + j] = t;
        }
    __syncthreads();
    if (threadIdx.x < kBL * kBL) {
        const int i = threadIdx.x / kBL, j = threadIdx.x % kBL;
        const int a = A * kBL + i, b = B * kBL + j;
        if (a < L && b < L && a < b) {
            float js = 0.f;
            for (int w = 0; w < kSimThreads / 64; ++w) js += part[w][threadIdx.x];
            const float s = 1.f - 0.5f * js / (float)R; // JS = (KL(p||m) + KL(q||m)) / 2, mean over the rows
            sim[((size_t)h * L + a) * L + b] = s;
            sim[((size_t)h * L + b) * L + a] = s;
        }
    }
}

__global__ void similarity_diagonal_kernel(int L, int H, float *__restrict__ sim)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < L * H) sim[((size_t)(i / L) * L + i % L) * L + i % L] = 1.f;
}

} // namespace

int pod_launch_similarity(const float *att, int L, int H, int R, int n, float *sim, hipStream_t st)
{
    hipLaunchKernelGGL(similarity_diagonal_kernel, dim3((L * H + 255) / 256), dim3(256), 0, st, L, H, sim);
    if (L > 1)
        hipLaunchKernelGGL(similarity_kernel, dim3((unsigned)(((L + kBL - 1) / kBL) * ((L + kBL - 1) / kBL + 1) / 2), (unsigned)H),
                           dim3(kSimThreads), 0, st, att, L, H, R, n, sim);
    POD_HIP_TRY(hipGetLastError());
    return POD_OK;
}
