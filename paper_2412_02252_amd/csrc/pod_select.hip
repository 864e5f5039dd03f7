// Token selection on the distant store: the combination of the cache with a token-selection method that the
// paper's result tables list as "PoD+SnapKV" (appendix section on SnapKV: an observation window of 64 prompt
// positions, extended to grouped-query attention).  The paper gives no rule of its own; what is computed here is
// the published selection rule on the part of the cache the combination can shrink, the distant tokens (the
// proximal ones are kept in full by definition, Section 3):
//
//   votes   vote[h][t] = sum over the last `obs` prompt positions i and over the query heads g of kv head h's group
//           of the attention weight that query (i, g) gives distant token t, in the joint softmax over the keys up
//           to position i (Eq. 4).  The call is made at a block's lowest layer, where every logit is that layer's
//           own q.k (Eq. 3) and the distant logits are the ones the whole block uses.
//   top     the votes are pooled over 2r+1 neighbours (mean with zeros outside the range, or maximum), the `keep`
//           largest per kv head are selected (of equal ones the earlier token), ascending.
//   compact per layer: the selected distant rows move to the front of the distant stores, the recent ring is
//           turned to where a sequence of S + keep + W tokens has it, and the stored length becomes that: the
//           cache is then the cache of the shorter sequence and every other call works on it unchanged.
//
// The votes are a dense contraction (obs * rep query rows x n keys x D per kv head) and run on
// v_mfma_f32_32x32x16_bf16 with both operands fetched from global memory in fragment order (a lane's fragment is 8
// consecutive bf16 of one row; the query rows of a kv head are 64 KB and stay in L2).  Two passes over the keys:
// the first takes each query row's maximum and sum of exponentials over all keys it sees (S^T = K Q^T: a lane
// owns a query row, so the reduction over keys is in-lane), the second recomputes the distant logits transposed
// (S = Q K^T: a lane owns a key, so the sum over query rows is in-lane) and writes one vote per key.  Every sum
// has a fixed order: the votes are reproducible bit for bit.
#include <math.h>

#include "pod_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 sel_bf16x8;
typedef __attribute__((ext_vector_type(16))) float sel_f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned sel_u32x4;

constexpr int kSelThreads = 256;        // 4 waves
constexpr int kSelKeysPerIter = 128;    // 32 keys per wave
constexpr int kTopThreads = 1024;
constexpr float kLog2e = 1.4426950408889634f;

struct select_params {
    const pod_bf16 *q_obs; // [obs][Hq][D]
    const pod_bf16 *k;     // [n][Hkv][D]
    int n, obs, Hq, Hkv, rep, S, W;
    int R;            // obs * rep query rows per kv head; row r = (position n - obs + r / rep, head h * rep + r % rep)
    int nrb;          // blocks of 32 rows
    int keys_per_wg;  // keys per workgroup of the first pass (a multiple of 128)
    int npieces;      // workgroups per kv head in the first pass
    float scale_log2; // logit scale times log2(e)
    uint64_t head_mask;
    float2 *part;     // [Hkv][npieces][nrb * 32]  (maximum, sum of exponentials) of a row over one piece of keys
    float2 *stat;     // [Hkv][nrb * 32]           (maximum, 1 / sum) over all keys the row sees
    float *votes;     // [Hkv][n - S - W]
};

// fragments of one row for all k-steps: 8 consecutive bf16 per k-step, at offset 8 * (lane / 32) inside the step
template <int D>
__device__ inline void load_row_fragments(const pod_bf16 *row, int lane, sel_u32x4 (&f)[D / 16])
{
    const sel_u32x4 *p = (const sel_u32x4 *)(row + 8 * (lane >> 5));
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) f[kk] = p[2 * kk];
}

__device__ inline const pod_bf16 *query_row(const select_params &p, int h, int r, int D)
{
    const int rr = r < p.R ? r : 0; // rows past the end read row 0 and are left out by the caller
    return p.q_obs + ((size_t)(rr / p.rep) * p.Hq + (size_t)h * p.rep + rr % p.rep) * D;
}

// (m, l) + (m2, l2) of two disjoint key sets; an empty set is (-inf, 0)
__device__ inline void merge_stat(float &m, float &l, float m2, float l2)
{
    const float M = fmaxf(m, m2);
    const float a = m > -INFINITY ? l * exp2f(m - M) : 0.f;
    const float b = m2 > -INFINITY ? l2 * exp2f(m2 - M) : 0.f;
    m = M;
    l = a + b;
}

template <int D>
__global__ __launch_bounds__(kSelThreads) void select_stat_kernel(select_params p)
{
    const int h = blockIdx.y;
    if (!((p.head_mask >> h) & 1)) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int key_lo = blockIdx.x * p.keys_per_wg;
    const int key_hi = key_lo + p.keys_per_wg < p.n ? key_lo + p.keys_per_wg : p.n;
    __shared__ float2 red[kSelThreads / 64][32];
    for (int rb = 0; rb < p.nrb; ++rb) {
        const int r = rb * 32 + (lane & 31);
        const int qpos = p.n - p.obs + (r < p.R ? r : 0) / p.rep; // the row's own position: it sees keys 0 .. qpos
        sel_u32x4 qf[D / 16];
        load_row_fragments<D>(query_row(p, h, r, D), lane, qf);
        float m = -INFINITY, l = 0.f;
        for (int key0 = key_lo + wave * 32; key0 < key_hi; key0 += kSelKeysPerIter) {
            const int key = key0 + (lane & 31) < p.n ? key0 + (lane & 31) : p.n - 1;
            sel_u32x4 kf[D / 16];
            load_row_fragments<D>(p.k + ((size_t)key * p.Hkv + h) * D, lane, kf);
            sel_f32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int kk = 0; kk < D / 16; ++kk)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(sel_bf16x8, kf[kk]),
                                                               __builtin_bit_cast(sel_bf16x8, qf[kk]), acc, 0, 0, 0);
            // accumulator e of this lane: key key0 + 8 (e / 4) + 4 (lane / 32) + e % 4, query row lane % 32
            float s[16], tmax = -INFINITY;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int ke = key0 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                s[e] = ke <= qpos ? acc[e] * p.scale_log2 : -INFINITY; // qpos < n: keys past the end drop out too
                tmax = fmaxf(tmax, s[e]);
            }
            if (tmax > -INFINITY) {
                const float mn = fmaxf(m, tmax);
                float add = 0.f;
#pragma unroll
                for (int e = 0; e < 16; ++e) add += exp2f(s[e] - mn);
                l = l * exp2f(m - mn) + add; // m = -inf: l is 0 and stays 0
                m = mn;
            }
        }
        merge_stat(m, l, __shfl_xor(m, 32), __shfl_xor(l, 32)); // the two lanes of a row hold different keys
        if (lane < 32) red[wave][lane] = make_float2(m, l);
        __syncthreads();
        if (threadIdx.x < 32) {
            float M = red[0][lane].x, L = red[0][lane].y;
            for (int w = 1; w < kSelThreads / 64; ++w) merge_stat(M, L, red[w][lane].x, red[w][lane].y);
            p.part[((size_t)h * p.npieces + blockIdx.x) * (p.nrb * 32) + r] = make_float2(M, L);
        }
        __syncthreads();
    }
}

__global__ void select_reduce_kernel(select_params p)
{
    const int h = blockIdx.y;
    if (!((p.head_mask >> h) & 1)) return;
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= p.nrb * 32) return;
    float M = -INFINITY, L = 0.f;
    for (int c = 0; c < p.npieces; ++c) {
        const float2 t = p.part[((size_t)h * p.npieces + c) * (p.nrb * 32) + r];
        merge_stat(M, L, t.x, t.y);
    }
    p.stat[(size_t)h * (p.nrb * 32) + r] = make_float2(M, L > 0.f ? 1.f / L : 0.f); // every row sees key 0: L > 0
}

template <int D>
__global__ __launch_bounds__(kSelThreads) void select_vote_kernel(select_params p)
{
    const int h = blockIdx.y;
    if (!((p.head_mask >> h) & 1)) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int dist_hi = p.n - p.W;                                         // distant keys: S .. n - W - 1
    const int key0 = p.S + blockIdx.x * kSelKeysPerIter + wave * 32;
    if (key0 >= dist_hi) return;                                           // (whole wave)
    const int key = key0 + (lane & 31) < dist_hi ? key0 + (lane & 31) : dist_hi - 1;
    sel_u32x4 kf[D / 16];
    load_row_fragments<D>(p.k + ((size_t)key * p.Hkv + h) * D, lane, kf);
    const float2 *stat = p.stat + (size_t)h * (p.nrb * 32);
    float vote = 0.f;
    for (int rb = 0; rb < p.nrb; ++rb) {
        sel_u32x4 qf[D / 16];
        load_row_fragments<D>(query_row(p, h, rb * 32 + (lane & 31), D), lane, qf);
        sel_f32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(sel_bf16x8, qf[kk]),
                                                           __builtin_bit_cast(sel_bf16x8, kf[kk]), acc, 0, 0, 0);
        // accumulator e of this lane: query row rb * 32 + 8 (e / 4) + 4 (lane / 32) + e % 4, key lane % 32; a distant
        // key is older than every query of the observation window (obs <= W), so no causal test is needed
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int r = rb * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
            if (r < p.R) {
                const float2 st = stat[r];
                vote += exp2f(acc[e] * p.scale_log2 - st.x) * st.y;
            }
        }
    }
    vote += __shfl_xor(vote, 32); // the two lanes of a key hold different query rows
    if (lane < 32 && key0 + lane < dist_hi) p.votes[(size_t)h * (dist_hi - p.S) + (key0 + lane - p.S)] = vote;
}

// order-preserving map of a float's bits to an unsigned (larger float = larger unsigned)
__device__ inline unsigned ordered_bits(float x)
{
    const unsigned u = __builtin_bit_cast(unsigned, x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// One workgroup per kv head: pool the votes, find the keep-th largest pooled vote by four rounds of 8-bit
// histograms over the ordered bit patterns, then write the indices of the selected tokens in ascending order
// (everything above the threshold, and the first `need` of those equal to it).
__global__ __launch_bounds__(kTopThreads) void select_top_kernel(const float *__restrict__ votes, int m, uint64_t head_mask,
                                                                 int width, int use_max, int keep, float *pooled,
                                                                 int32_t *sel, int sel_stride)
{
    const int h = blockIdx.x;
    if (!((head_mask >> h) & 1)) return;
    const float *v = votes + (size_t)h * m;
    float *pl = pooled + (size_t)h * m;
    int32_t *out = sel + (size_t)h * sel_stride;
    const int tid = threadIdx.x, r = width / 2;
    for (int t = tid; t < m; t += kTopThreads) {
        const int lo = t - r > 0 ? t - r : 0, hi = t + r + 1 < m ? t + r + 1 : m;
        float x;
        if (use_max) {
            x = v[lo];
            for (int u = lo + 1; u < hi; ++u) x = fmaxf(x, v[u]);
        } else {
            float acc = 0.f;
            for (int u = lo; u < hi; ++u) acc = acc + v[u];
            x = acc / (float)width;
        }
        pl[t] = x;
    }
    __shared__ unsigned hist[256];
    __shared__ unsigned s_prefix, s_need;
    __shared__ unsigned wave_tot[kTopThreads / 64];
    if (tid == 0) { s_prefix = 0; s_need = (unsigned)keep; }
    __syncthreads();
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        const unsigned prefix = s_prefix;
        for (int t = tid; t < m; t += kTopThreads) {
            const unsigned key = ordered_bits(pl[t]);
            if (shift == 24 || (key >> (shift + 8)) == (prefix >> (shift + 8))) atomicAdd(&hist[(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid == 0) {
            unsigned need = s_need;
            int d = 255;
            for (; d > 0; --d) { // the digit whose bucket holds the need-th largest of the candidates
                if (hist[d] >= need) break;
                need -= hist[d];
            }
            s_prefix = prefix | ((unsigned)d << shift);
            s_need = need;
        }
        __syncthreads();
    }
    const unsigned thr = s_prefix, need = s_need; // need >= 1 entries equal to the threshold are taken, earliest first
    unsigned run_gt = 0, run_eq = 0;
    const int lane = tid & 63, wave = tid >> 6;
    for (int base = 0; base < m; base += kTopThreads) {
        const int t = base + tid;
        const unsigned key = t < m ? ordered_bits(pl[t]) : 0u;
        const bool gt = t < m && key > thr, eq = t < m && key == thr;
        const unsigned long long bg = __ballot(gt), be = __ballot(eq), below = (1ull << lane) - 1ull;
        if (lane == 0) wave_tot[wave] = (unsigned)__popcll(bg) | ((unsigned)__popcll(be) << 16);
        __syncthreads();
        unsigned before = 0, total = 0;
        for (int w = 0; w < kTopThreads / 64; ++w) {
            if (w < wave) before += wave_tot[w];
            total += wave_tot[w];
        }
        const unsigned gt_before = run_gt + (before & 0xFFFFu) + (unsigned)__popcll(bg & below);
        const unsigned eq_before = run_eq + (before >> 16) + (unsigned)__popcll(be & below);
        if (gt || (eq && eq_before < need)) {
            const unsigned pos = gt_before + (eq_before < need ? eq_before : need);
            if (pos < (unsigned)keep) out[pos] = t;
        }
        run_gt += total & 0xFFFFu;
        run_eq += total >> 16;
        __syncthreads();
    }
}

struct compact_params {
    char *base;
    pod_layout ly;
    pod_headmap hm;
    int layer, b, n, keep;
    const int32_t *sel_all;           // [L][Hkv][keep]
    int32_t sel_layer[kMaxKvHeads];   // the lowest layer of kv head h's block: whose selection h follows here
    uint4 *ws;                        // [2][Hkv][keep + W][D] bf16: rows on their way (keys, then values)
};

// stage 0 copies the surviving rows into the workspace, stage 1 copies them back to where the shorter sequence
// keeps them; both do nothing unless the stored length is n (compact_commit_kernel then raises the flag).
// Rows 0 .. keep - 1: selected distant rows; rows keep .. keep + W - 1: the recent window, oldest first.
template <int STAGE>
__global__ void compact_move_kernel(compact_params p)
{
    const pod_layout &ly = p.ly;
    const int32_t *lens = (const int32_t *)(p.base + ly.off_lens);
    if (lens[(size_t)p.layer * ly.B + p.b] != p.n) return;
    const int h = blockIdx.y, is_v = blockIdx.z;
    const int cpr = ly.D / 8, rows = p.keep + ly.W, n_dist = p.n - ly.S - ly.W;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= rows * cpr) return;
    const int row = idx / cpr, c = idx % cpr;
    const bool low = (p.hm.lowest_mask >> h) & 1;
    uint4 *wsrow = p.ws + (((size_t)is_v * ly.Hkv + h) * rows + row) * cpr + c;
    uint4 *cache_row;
    if (row < p.keep) {
        if (!is_v && !low) return; // this layer keeps no distant keys for head h
        size_t r = row;
        if (STAGE == 0) {
            const int t = p.sel_all[((size_t)p.sel_layer[h] * ly.Hkv + h) * p.keep + row];
            if (t < 0 || t >= n_dist) {
                atomicOr((int32_t *)(p.base + ly.off_flag), 1); // not a selection: copy row 0, report
                r = 0;
            } else {
                r = (size_t)t;
            }
        }
        cache_row = is_v ? (uint4 *)(p.base + ly.off_distV) + (pod_dist_row0(ly, p.layer, p.b, h) + r) * cpr + c
                         : (uint4 *)(p.base + ly.off_distK) + (pod_distk_row0(ly, p.hm, p.b, h) + r) * cpr + c;
    } else {
        const int i = row - p.keep; // position n - W + i before, S + keep + i after
        const int slot = ly.S + (STAGE == 0 ? (p.n - ly.S + i) % ly.W : (p.keep + i) % ly.W);
        cache_row = (uint4 *)(p.base + (is_v ? ly.off_proxV : ly.off_proxK)) + (pod_prox_row0(ly, p.layer, p.b, h) + slot) * cpr + c;
    }
    if (STAGE == 0) *wsrow = *cache_row;
    else *cache_row = *wsrow;
}

__global__ void compact_commit_kernel(char *base, pod_layout ly, int layer, int b, int n, int n_new)
{
    int32_t *len = (int32_t *)(base + ly.off_lens) + (size_t)layer * ly.B + b;
    if (*len == n) *len = n_new;
    else atomicOr((int32_t *)(base + ly.off_flag), 1);
}

inline size_t up256(size_t x) { return (x + 255) / 256 * 256; }

struct select_plan { int R, nrb, keys_per_wg, npieces; size_t off_stat, bytes; };

select_plan plan_votes(const pod_layout &ly, int64_t n, int obs)
{
    select_plan s;
    s.R = obs * ly.rep;
    s.nrb = (s.R + 31) / 32;
    int per = (int)((n + 63) / 64);
    s.keys_per_wg = (per + kSelKeysPerIter - 1) / kSelKeysPerIter * kSelKeysPerIter;
    s.npieces = (int)((n + s.keys_per_wg - 1) / s.keys_per_wg);
    s.off_stat = up256((size_t)ly.Hkv * s.npieces * s.nrb * 32 * sizeof(float2));
    s.bytes = s.off_stat + up256((size_t)ly.Hkv * s.nrb * 32 * sizeof(float2));
    return s;
}

} // namespace

size_t pod_select_votes_bytes(const pod_layout &ly, int64_t n, int obs) { return plan_votes(ly, n, obs).bytes; }
size_t pod_select_top_bytes(const pod_layout &ly, int64_t n) { return up256((size_t)ly.Hkv * (size_t)(n - ly.S - ly.W) * sizeof(float)); }
size_t pod_compact_bytes(const pod_layout &ly, int keep) { return up256((size_t)2 * ly.Hkv * ((size_t)keep + ly.W) * ly.D * 2); }

int pod_launch_select_votes(const pod_layout &ly, uint64_t head_mask, int n, const void *q_obs, int obs, const void *k,
                            float scale, float *votes, void *ws, hipStream_t st)
{
    const select_plan s = plan_votes(ly, n, obs);
    select_params p;
    p.q_obs = (const pod_bf16 *)q_obs; p.k = (const pod_bf16 *)k;
    p.n = n; p.obs = obs; p.Hq = ly.Hq; p.Hkv = ly.Hkv; p.rep = ly.rep; p.S = ly.S; p.W = ly.W;
    p.R = s.R; p.nrb = s.nrb; p.keys_per_wg = s.keys_per_wg; p.npieces = s.npieces;
    p.scale_log2 = scale * kLog2e;
    p.head_mask = head_mask;
    p.part = (float2 *)ws; p.stat = (float2 *)((char *)ws + s.off_stat); p.votes = votes;
    const int n_dist = n - ly.S - ly.W;
    const dim3 g1(s.npieces, ly.Hkv), g2((s.nrb * 32 + 255) / 256, ly.Hkv), g3((n_dist + kSelKeysPerIter - 1) / kSelKeysPerIter, ly.Hkv);
    if (ly.D == 128) {
        hipLaunchKernelGGL(select_stat_kernel<128>, g1, dim3(kSelThreads), 0, st, p);
        hipLaunchKernelGGL(select_reduce_kernel, g2, dim3(256), 0, st, p);
        hipLaunchKernelGGL(select_vote_kernel<128>, g3, dim3(kSelThreads), 0, st, p);
    } else {
        hipLaunchKernelGGL(select_stat_kernel<64>, g1, dim3(kSelThreads), 0, st, p);
        hipLaunchKernelGGL(select_reduce_kernel, g2, dim3(256), 0, st, p);
        hipLaunchKernelGGL(select_vote_kernel<64>, g3, dim3(kSelThreads), 0, st, p);
    }
    POD_HIP_TRY(hipGetLastError());
    return POD_OK;
}

int pod_launch_select_top(int Hkv, uint64_t head_mask, const float *votes, int m, int width, int use_max, int keep,
                          float *pooled, int32_t *sel, int sel_stride, hipStream_t st)
{
    hipLaunchKernelGGL(select_top_kernel, dim3(Hkv), dim3(kTopThreads), 0, st, votes, m, head_mask, width, use_max, keep, pooled,
                       sel, sel_stride);
    POD_HIP_TRY(hipGetLastError());
    return POD_OK;
}

int pod_launch_compact(const pod_cache *c, int layer, int b, int n, const int32_t *sel_all, int keep, void *ws, hipStream_t st)
{
    const pod_layout &ly = c->ly;
    compact_params p;
    p.base = c->base; p.ly = ly; p.hm = pod_make_headmap(c, layer);
    p.layer = layer; p.b = b; p.n = n; p.keep = keep; p.sel_all = sel_all; p.ws = (uint4 *)ws;
    for (int h = 0; h < ly.Hkv; ++h) p.sel_layer[h] = c->lowest[(size_t)layer * ly.Hkv + h];
    const int items = (keep + ly.W) * (ly.D / 8);
    const dim3 g((items + 255) / 256, ly.Hkv, 2);
    hipLaunchKernelGGL(compact_move_kernel<0>, g, dim3(256), 0, st, p);
    hipLaunchKernelGGL(compact_move_kernel<1>, g, dim3(256), 0, st, p);
    hipLaunchKernelGGL(compact_commit_kernel, dim3(1), dim3(1), 0, st, c->base, ly, layer, b, n, ly.S + keep + ly.W);
    POD_HIP_TRY(hipGetLastError());
    return POD_OK;
}
