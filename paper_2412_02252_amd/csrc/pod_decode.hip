// Decode attention over the split cache: split-K flash decoding on gfx950.
//
// One query token per sequence (Eq. 3 of the paper with i = n-1) and one joint softmax over
// proximal and distant tokens (Eq. 4 / appendix derivation).  The token axis of every
// (sequence, kv head) pair is cut in chunks; a workgroup reduces one chunk to a partial
// (running max m, normaliser l, unnormalised output acc) and a second kernel merges the
// partials.  The merge of two partials is exactly the paper's gate: with l_P, l_D the two
// normalisers brought to a common max, g = l_P / (l_P + l_D).
//
// The kernel is bound by streaming K and V rows from HBM once, so the design goals are
// (1) every global load instruction reads whole contiguous rows, (2) enough loads in flight
// per wave, (3) arithmetic stays off the critical path.  The (Hq/Hkv <= 16) query heads that
// share a kv head are padded to a 16-wide MFMA operand so both products run on the matrix
// cores:
//   S^T[token][head] = K[token][:] . Q[head][:]        v_mfma_f32_16x16x32_bf16, A = K, B = Q
//   O^T[dim][head]   = sum_token V[token][dim] P[token][head]            A = V^T, B = P
// With head as the MFMA column (lane % 16) in both products, every lane owns one head's
// softmax state and that head's slice of the output: no cross-lane traffic except the
// 4-lane max/sum reductions.
//
// Operand layouts (lane = 16*j + m, the lane holds 8 consecutive k-values 8j..8j+7):
//  * K as A operand needs lane (m, j) to hold 16 bytes of token m.  Rows are loaded fully
//    coalesced (16 lanes per 256-byte row) and turned through a per-wave LDS tile with an
//    XOR swizzle.
//  * V^T as A operand needs 8 *tokens* of one dim per lane.  Each lane loads the same
//    16-byte dim chunk of 8 different tokens (each load instruction still reads whole rows)
//    and transposes the 8x8 block in registers (v_perm_b32).  The MFMA k-index is only a
//    summation index, so the 8 tokens a lane holds are chosen to be exactly the 8 tokens
//    whose probabilities the same lane already holds in the S^T accumulators of two
//    16-token MFMA tiles: tokens {4j..4j+3} of tile 0 and of tile 1.
#include "pod_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4; // native 128-bit vector (plain loads/stores, no struct copies)

constexpr int kWaves = 4;          // waves per workgroup
constexpr int kTile = 32;          // tokens per wave iteration
constexpr float kNegBig = -1.0e30f; // stands in for -inf (keeps exp2 arguments finite)
constexpr int kMinChunk = 128;     // smallest chunk (tokens) a workgroup takes

struct decode_params {
    const char *base;
    pod_layout ly;
    int layer, B;
    const pod_bf16 *q, *q_shared;
    const int32_t *ctx;
    float scale_log2e;
    int chunk;   // tokens per workgroup
    int max_nd;  // distant chunk slots per (sequence, head)
    int max_np;  // proximal chunk slots
    float *part_acc; // [B][Hq][NC][D]
    float *part_ml;  // [B][Hq][NC][2]
    pod_bf16 *out;   // [B][Hq][D]
};

// Length of sequence b as the decode kernels see it: 0 = skip (inactive, or contract
// violated: then *bad is set).  Also requires the block's lowest layer to be in step.
__device__ inline int decode_seq_len(const decode_params &p, int b, bool *bad)
{
    const int32_t *lens = (const int32_t *)(p.base + p.ly.off_lens);
    const int n = p.ctx[b];
    *bad = false;
    if (n == 0) return 0;
    const int lowest = p.layer - p.layer % p.ly.G;
    if (n < 0 || n > p.ly.maxctx || n != lens[(size_t)p.layer * p.ly.B + b] ||
        (n > p.ly.P && lens[(size_t)lowest * p.ly.B + b] != n)) {
        *bad = true;
        return 0;
    }
    return n;
}

__device__ inline bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ inline unsigned pack_bf16(float lo, float hi)
{
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    bf16x2 t = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(unsigned, t);
}

template <int D>
__global__ __launch_bounds__(kWaves * 64) void decode_partial_kernel(decode_params p)
{
    constexpr int CPR = D / 8;        // 16-byte pieces per row
    constexpr int RPI = 64 / CPR;     // rows one K load instruction covers
    constexpr int NLD = kTile / RPI;  // K load instructions per tile
    constexpr int KST = D / 32;       // MFMA k-steps over the head dim
    constexpr int XN = 16 / CPR;      // lanes sharing one V piece (1 for D=128, 2 for D=64)
    constexpr int NPV = 8 / XN;       // PV MFMAs per tile

    const pod_layout &ly = p.ly;
    const int b = blockIdx.z, h = blockIdx.y, c = blockIdx.x;
    bool bad;
    const int n = decode_seq_len(p, b, &bad);
    if (n == 0) return; // the combine kernel zeroes the output and raises the flag
    const int n_prox = n < ly.P ? n : ly.P;
    const int n_dist = n - n_prox;
    const bool distant = c < p.max_nd;
    const int region_len = distant ? n_dist : n_prox;
    const int start = (distant ? c : c - p.max_nd) * p.chunk;
    if (start >= region_len) return;
    const int end = min(start + p.chunk, region_len);

    const int group = p.layer / ly.G;
    const u32x4 *Kb = distant ? (const u32x4 *)(p.base + ly.off_distK) + pod_dist_row0(ly, group, b, h) * CPR
                              : (const u32x4 *)(p.base + ly.off_proxK) + pod_prox_row0(ly, p.layer, b, h) * CPR;
    const u32x4 *Vb = distant ? (const u32x4 *)(p.base + ly.off_distV) + pod_dist_row0(ly, p.layer, b, h) * CPR
                              : (const u32x4 *)(p.base + ly.off_proxV) + pod_prox_row0(ly, p.layer, b, h) * CPR;
    const pod_bf16 *qsrc = (distant && p.q_shared) ? p.q_shared : p.q;

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int m16 = lane & 15, j = lane >> 4;

    // kWaves K tiles of kTile rows; the same bytes later hold the merge buffer
    // [kWaves][rep <= 16][D] floats, which is exactly as large.
    __shared__ u32x4 lds[kWaves][kTile * CPR];
    static_assert(sizeof(u32x4) * kTile * CPR == sizeof(float) * 16 * D, "merge buffer must fit the K tiles");
    u32x4 *ldsK = lds[wave];

    // Q as B operand: lane (head m16, j) holds dims 32s + 8j .. +7 of its head (zero past rep).
    bf16x8 qf[KST];
    {
        const u32x4 *qrow = (const u32x4 *)(qsrc + ((size_t)b * ly.Hq + (size_t)h * ly.rep + m16) * D);
#pragma unroll
        for (int s = 0; s < KST; ++s) {
            u32x4 t = u32x4{0u, 0u, 0u, 0u};
            if (m16 < ly.rep) t = qrow[4 * s + j];
            qf[s] = as_bf16x8(t);
        }
    }

    f32x4 acc[NPV];
#pragma unroll
    for (int x = 0; x < NPV; ++x) acc[x] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = kNegBig, l_run = 0.f;

    const int kr = lane / CPR, kc = lane % CPR; // K load: row within the instruction, piece
    const int vc = lane % CPR;                  // V load: piece
    const int vx = (lane / CPR) % XN;           // which of the XN dims per piece pair this lane serves
    const int last = end - 1;

    // Tile loads.  Rows past the chunk are clamped to its last row (valid memory, masked later),
    // so the loads are unconditional: the software pipeline below needs no branches around them.
    u32x4 kreg[NLD], vreg[8];
#define POD_LOAD_TILE(T0)                                                         \
    _Pragma("unroll") for (int i = 0; i < NLD; ++i) {                             \
        const int row = min((T0) + RPI * i + kr, last);                           \
        kreg[i] = Kb[(size_t)row * CPR + kc];                                     \
    }                                                                             \
    _Pragma("unroll") for (int e = 0; e < 8; ++e) {                               \
        const int tok = (e < 4) ? 4 * j + e : 16 + 4 * j + (e - 4);               \
        const int row = min((T0) + tok, last);                                    \
        vreg[e] = Vb[(size_t)row * CPR + vc];                                     \
    }

    int t0 = start + wave * kTile;
    POD_LOAD_TILE(t0)

    for (; t0 < end; t0 += kWaves * kTile) {
        // ---- K tile through LDS into A-operand order
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int r = RPI * i + kr;
            ldsK[r * CPR + (kc ^ (r % CPR))] = kreg[i];
        }
        u32x4 vcur[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) vcur[e] = vreg[e];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();

        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KST; ++s) {
            const int col = 4 * s + j;
            const u32x4 a0 = ldsK[m16 * CPR + (col ^ (m16 % CPR))];
            const u32x4 a1 = ldsK[(16 + m16) * CPR + (col ^ ((16 + m16) % CPR))];
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a0), qf[s], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a1), qf[s], s1, 0, 0, 0);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();

        // ---- next tile's loads go out before the softmax / PV work of this one
        POD_LOAD_TILE(t0 + kWaves * kTile)

        // ---- online softmax for head m16 over this lane's 8 tokens (base-2 domain)
        float sc[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int tok0 = t0 + 4 * j + i, tok1 = tok0 + 16;
            sc[i] = tok0 < end ? s0[i] * p.scale_log2e : kNegBig;
            sc[4 + i] = tok1 < end ? s1[i] * p.scale_log2e : kNegBig;
        }
        float mx = sc[0];
#pragma unroll
        for (int i = 1; i < 8; ++i) mx = fmaxf(mx, sc[i]);
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = exp2f(m_run - m_new);
        float ps = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) { sc[i] = exp2f(sc[i] - m_new); ps += sc[i]; }
        ps += __shfl_xor(ps, 16);
        ps += __shfl_xor(ps, 32);
        l_run = l_run * alpha + ps;
        m_run = m_new;
#pragma unroll
        for (int x = 0; x < NPV; ++x) acc[x] *= alpha;
        u32x4 pw;
        pw.x = pack_bf16(sc[0], sc[1]); pw.y = pack_bf16(sc[2], sc[3]);
        pw.z = pack_bf16(sc[4], sc[5]); pw.w = pack_bf16(sc[6], sc[7]);
        const bf16x8 pf = as_bf16x8(pw);

        // ---- V: 8x8 in-register transpose, then O^T += V^T P
        // vcur[e] = dims 8*vc .. +7 of token e (of this lane's 8); want per dim the 8 tokens.
#pragma unroll
        for (int x = 0; x < NPV; ++x) {
            // dim index inside the piece: XN = 1 -> x ; XN = 2 -> 2x + vx
            u32x4 tlo, thi; // candidates for the even / odd dim of dword pair
            const int w = (XN == 1) ? (x >> 1) : x; // dword of the piece holding the dim(s)
            auto dw = [&](const u32x4 &u) -> unsigned { return u[w]; };
            tlo.x = __builtin_amdgcn_perm(dw(vcur[1]), dw(vcur[0]), 0x05040100u);
            tlo.y = __builtin_amdgcn_perm(dw(vcur[3]), dw(vcur[2]), 0x05040100u);
            tlo.z = __builtin_amdgcn_perm(dw(vcur[5]), dw(vcur[4]), 0x05040100u);
            tlo.w = __builtin_amdgcn_perm(dw(vcur[7]), dw(vcur[6]), 0x05040100u);
            thi.x = __builtin_amdgcn_perm(dw(vcur[1]), dw(vcur[0]), 0x07060302u);
            thi.y = __builtin_amdgcn_perm(dw(vcur[3]), dw(vcur[2]), 0x07060302u);
            thi.z = __builtin_amdgcn_perm(dw(vcur[5]), dw(vcur[4]), 0x07060302u);
            thi.w = __builtin_amdgcn_perm(dw(vcur[7]), dw(vcur[6]), 0x07060302u);
            u32x4 vt;
            if (XN == 1) {
                vt = (x & 1) ? thi : tlo;
            } else {
                vt.x = vx ? thi.x : tlo.x; vt.y = vx ? thi.y : tlo.y;
                vt.z = vx ? thi.z : tlo.z; vt.w = vx ? thi.w : tlo.w;
            }
            acc[x] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(vt), pf, acc[x], 0, 0, 0);
        }
    }

#undef POD_LOAD_TILE
    // ---- merge the waves of this workgroup, write one partial per (head, chunk)
    // acc[x][i] is O^T[dim slot 4j+i][head m16]; the slot's dim is
    //   XN = 1: 8*(4j+i) + x        XN = 2: 8*((4j+i) % 8) + 2x + (4j+i)/8
    __syncthreads(); // all waves are done with their K tiles
    float *sm_acc = (float *)&lds[0][0];              // [kWaves][rep][D]
    __shared__ float sm_m[kWaves][16], sm_l[kWaves][16];
    if (m16 < ly.rep) {
#pragma unroll
        for (int x = 0; x < NPV; ++x)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int slot = 4 * j + i;
                const int dim = (XN == 1) ? 8 * slot + x : 8 * (slot % 8) + 2 * x + slot / 8;
                sm_acc[((size_t)wave * ly.rep + m16) * D + dim] = acc[x][i];
            }
        if (j == 0) { sm_m[wave][m16] = m_run; sm_l[wave][m16] = l_run; }
    }
    __syncthreads();
    const int NC = p.max_nd + p.max_np;
    for (int t = threadIdx.x; t < ly.rep * D; t += blockDim.x) {
        const int head = t / D, dim = t % D;
        float M = sm_m[0][head];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) M = fmaxf(M, sm_m[w][head]);
        float A = 0.f, Lsum = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float f = exp2f(sm_m[w][head] - M);
            A += f * sm_acc[((size_t)w * ly.rep + head) * D + dim];
            Lsum += f * sm_l[w][head];
        }
        const size_t slot = ((size_t)b * ly.Hq + (size_t)h * ly.rep + head) * NC + c;
        p.part_acc[slot * D + dim] = A;
        if (dim == 0) { p.part_ml[slot * 2] = M; p.part_ml[slot * 2 + 1] = Lsum; }
    }
}

// One workgroup per (query head, sequence): merge the chunk partials, normalise, round to bf16.
template <int D>
__global__ __launch_bounds__(256) void decode_combine_kernel(decode_params p)
{
    constexpr int LPR = D / 4;       // lanes per partial row (float4 each)
    constexpr int NG = 256 / LPR;    // chunk groups
    const pod_layout &ly = p.ly;
    const int head = blockIdx.x, b = blockIdx.y;
    bool bad;
    const int n = decode_seq_len(p, b, &bad);
    pod_bf16 *orow = p.out + ((size_t)b * ly.Hq + head) * D;
    if (n == 0) {
        if (bad && head == 0 && threadIdx.x == 0) atomicOr((int32_t *)(p.base + ly.off_flag), 2);
        for (int t = threadIdx.x; t < D; t += blockDim.x) orow[t] = 0;
        return;
    }
    const int n_prox = n < ly.P ? n : ly.P;
    const int n_dist = n - n_prox;
    const int nd = (n_dist + p.chunk - 1) / p.chunk;
    const int np = (n_prox + p.chunk - 1) / p.chunk;
    const int NC = p.max_nd + p.max_np;
    const int nvalid = nd + np;
    const float *ml = p.part_ml + ((size_t)b * ly.Hq + head) * NC * 2;
    const float4 *pa = (const float4 *)(p.part_acc + ((size_t)b * ly.Hq + head) * NC * D);
    auto chunk_slot = [&](int v) { return v < nd ? v : p.max_nd + (v - nd); };

    __shared__ float red[256];
    float mx = kNegBig;
    for (int v = threadIdx.x; v < nvalid; v += 256) mx = fmaxf(mx, ml[chunk_slot(v) * 2]);
    red[threadIdx.x] = mx;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (threadIdx.x < s) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + s]);
        __syncthreads();
    }
    const float M = red[0];
    __syncthreads();

    const int g = threadIdx.x / LPR, x = threadIdx.x % LPR;
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
    float lsum = 0.f;
    for (int v = g; v < nvalid; v += NG) {
        const int cs = chunk_slot(v);
        const float f = exp2f(ml[cs * 2] - M);
        const float4 t = pa[(size_t)cs * LPR + x];
        a.x += f * t.x; a.y += f * t.y; a.z += f * t.z; a.w += f * t.w;
        lsum += f * ml[cs * 2 + 1];
    }
    __shared__ float4 sa[NG][LPR];
    __shared__ float sl[NG];
    sa[g][x] = a;
    if (x == 0) sl[g] = lsum;
    __syncthreads();
    if (g == 0) {
        float L = sl[0];
        for (int k = 1; k < NG; ++k) {
            const float4 t = sa[k][x];
            a.x += t.x; a.y += t.y; a.z += t.z; a.w += t.w;
            L += sl[k];
        }
        const float inv = 1.f / L;
        uint2 o;
        o.x = pack_bf16(a.x * inv, a.y * inv);
        o.y = pack_bf16(a.z * inv, a.w * inv);
        ((uint2 *)orow)[x] = o;
    }
}

int chunk_slots(int rows, int chunk) { return (rows + chunk - 1) / chunk; }

} // namespace

size_t pod_decode_workspace_bytes(const pod_layout &ly)
{
    const size_t nc = (size_t)chunk_slots(ly.Cd, kMinChunk) + chunk_slots(ly.P, kMinChunk) + 2;
    const size_t bytes = (size_t)ly.B * ly.Hq * nc * (ly.D + 2) * sizeof(float);
    return (bytes + 255) / 256 * 256;
}

int pod_launch_decode(const pod_cache *c, int layer, const void *q, const void *q_shared, const int32_t *ctx, int B,
                      int max_len, float scale, void *ws, size_t ws_bytes, void *out, hipStream_t st)
{
    const pod_layout &ly = c->ly;
    decode_params p;
    p.base = c->base; p.ly = ly; p.layer = layer; p.B = B;
    p.q = (const pod_bf16 *)q; p.q_shared = (const pod_bf16 *)q_shared; p.ctx = ctx;
    p.scale_log2e = scale * 1.4426950408889634f;
    p.out = (pod_bf16 *)out;

    // Chunk size: enough workgroups to fill 256 CUs a few times over, but no smaller than
    // kMinChunk tokens so the partials stay a small fraction of the K/V bytes.
    const char *env = getenv("POD_DECODE_CHUNK"); // tuning / test override
    const int env_chunk = env ? atoi(env) : 0;
    const long rows = (long)max_len * ly.Hkv * B;
    long chunk = env_chunk > 0 ? env_chunk : rows / 1024;
    chunk = (chunk + kMinChunk - 1) / kMinChunk * kMinChunk;
    if (chunk < kMinChunk) chunk = kMinChunk;
    if (chunk > 8192) chunk = 8192;
    p.chunk = (int)chunk;
    const int max_prox = max_len < ly.P ? max_len : ly.P;
    const int max_dist = max_len - max_prox;
    p.max_nd = chunk_slots(max_dist, p.chunk);
    p.max_np = chunk_slots(max_prox, p.chunk);
    const size_t NC = (size_t)p.max_nd + p.max_np;
    const size_t acc_bytes = (size_t)B * ly.Hq * NC * ly.D * sizeof(float);
    const size_t ml_bytes = (size_t)B * ly.Hq * NC * 2 * sizeof(float);
    if (acc_bytes + ml_bytes > ws_bytes) return pod_fail(POD_ERR_CAPACITY, "decode workspace too small");
    p.part_acc = (float *)ws;
    p.part_ml = (float *)((char *)ws + acc_bytes);

    const dim3 grid((unsigned)NC, (unsigned)ly.Hkv, (unsigned)B);
    const dim3 cgrid((unsigned)ly.Hq, (unsigned)B);
    pod_cache *mc = const_cast<pod_cache *>(c);
    const bool prof = mc->prof_ev && mc->prof_n < mc->prof_cap;
    if (prof) POD_HIP_TRY(hipEventRecord(mc->prof_ev[2 * mc->prof_n], st));
    if (ly.D == 128)
        hipLaunchKernelGGL(decode_partial_kernel<128>, grid, dim3(kWaves * 64), 0, st, p);
    else
        hipLaunchKernelGGL(decode_partial_kernel<64>, grid, dim3(kWaves * 64), 0, st, p);
    if (prof) { POD_HIP_TRY(hipEventRecord(mc->prof_ev[2 * mc->prof_n + 1], st)); mc->prof_n += 1; }
    if (ly.D == 128)
        hipLaunchKernelGGL(decode_combine_kernel<128>, cgrid, dim3(256), 0, st, p);
    else
        hipLaunchKernelGGL(decode_combine_kernel<64>, cgrid, dim3(256), 0, st, p);
    POD_HIP_TRY(hipGetLastError());
    return POD_OK;
}
