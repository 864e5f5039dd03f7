// Inter-layer attention similarity for the offline layer grouping (the paper's "Attention Similarity
// Measurement"): for head h and layers a, b, the Jensen-Shannon divergence of the two layers' attention
// rows, averaged over the sampled rows; the similarity is 1 minus that average with base-2 logarithms
// (base-2 JS lies in [0, 1], so identical rows give 1 and rows with disjoint support give 0).
//
// Memory-bound elementwise work followed by a reduction: one workgroup per (layer pair a < b, head)
// streams the two layers' rows once, 16 bytes per lane and load.  Nothing here is on the inference
// path; it feeds pod_group_layers.
#include "pod_internal.h"

namespace {

constexpr int kSimThreads = 256;

// p log2(p / m) + q log2(q / m) with m = (p + q) / 2 and 0 log 0 = 0
__device__ inline float js_term(float p, float q)
{
    const float m = 0.5f * (p + q);
    const float lm = __log2f(m);
    // (subnormal probabilities count as 0: the hardware logarithm flushes them, and x log x < 1e-35 there)
    constexpr float kMinNormal = 1.17549435e-38f;
    float t = 0.f;
    if (p >= kMinNormal) t += p * (__log2f(p) - lm);
    if (q >= kMinNormal) t += q * (__log2f(q) - lm);
    return t;
}

// att: [L][H][R][n] probabilities (rows sum to 1); sim: [H][L][L]
__global__ __launch_bounds__(kSimThreads) void similarity_kernel(const float *__restrict__ att, int L, int H, int R, int n,
                                                                 float *__restrict__ sim)
{
    // pair index -> (a, b), a < b
    int a = 0, rem = blockIdx.x;
    while (rem >= L - 1 - a) { rem -= L - 1 - a; ++a; }
    const int b = a + 1 + rem, h = blockIdx.y;
    const size_t rows = (size_t)R * n; // the R rows of one (layer, head) are contiguous
    const float *pa = att + ((size_t)a * H + h) * rows;
    const float *pb = att + ((size_t)b * H + h) * rows;
    float acc = 0.f;
    const size_t vec = rows / 4;
    for (size_t i = threadIdx.x; i < vec; i += kSimThreads) {
        const float4 x = ((const float4 *)pa)[i], y = ((const float4 *)pb)[i];
        acc += js_term(x.x, y.x) + js_term(x.y, y.y) + js_term(x.z, y.z) + js_term(x.w, y.w);
    }
    for (size_t i = vec * 4 + threadIdx.x; i < rows; i += kSimThreads) acc += js_term(pa[i], pb[i]);
    // workgroup reduction
    __shared__ float part[kSimThreads / 64];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        float js = 0.f;
        for (int w = 0; w < kSimThreads / 64; ++w) js += part[w];
        const float s = 1.f - 0.5f * js / (float)R; // JS = (KL(p||m) + KL(q||m)) / 2, mean over the rows
        sim[((size_t)h * L + a) * L + b] = s;
        sim[((size_t)h * L + b) * L + a] = s;
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
        hipLaunchKernelGGL(similarity_kernel, dim3((unsigned)(L * (L - 1) / 2), (unsigned)H), dim3(kSimThreads), 0, st, att, L, H, R, n, sim);
    POD_HIP_TRY(hipGetLastError());
    return POD_OK;
}
