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
// v_mfma_f32_32x32x16_bf16: the query rows of a kv head (64 KB at 64 positions x 4 heads x 128) are staged in LDS,
// the keys come from global memory in fragment order (a lane's fragment is 8 consecutive bf16 of one row) once per
// workgroup, and every key fragment meets all row blocks out of LDS.  Two passes over the keys:
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
    const pod_bf16 *k;     // [n][Hkv][D], or NULL: the keys are read where the cache holds them (below)
    // per kv head, in bf16 elements from the cache buffer's start: row 0 of the head's sink + ring rows and of the
    // distant-key store it reads at this layer (which is its own: the call is made at the block's lowest layer)
    const pod_bf16 *cache_base;
    unsigned long long prox0[kMaxKvHeads], dist0[kMaxKvHeads];
    int n, obs, Hq, Hkv, rep, S, W;
    int R;            // obs * rep query rows per kv head; row r = (position n - obs + r / rep, head h * rep + r % rep)
    int nrb;          // blocks of 32 rows
    int keys_per_wg;  // keys per workgroup of the first pass (a multiple of 128)
    int npieces;      // workgroups per kv head in the first pass
    float scale_log2; // logit scale times log2(e)
    uint64_t head_mask;
    float2 *part;     // [Hkv][npieces][nrb * 32]  (maximum, sum of exponentials) of a row over one piece of keys
    float *stat;      // [Hkv][nrb * 32]           maximum + log2(sum of exponentials) over all keys the row sees
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

// v_exp_f32: 2^x to 1 ulp; results below the smallest normal number come out as 0, which a softmax weight may
__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// where the key of position `key` of kv head h is: in the caller's array, or in the cache (sink slot, distant row,
// or the ring slot of a recent position)
__device__ inline const pod_bf16 *key_address(const select_params &p, int h, int key, int D)
{
    if (p.k) return p.k + ((size_t)key * p.Hkv + h) * D;
    if (key < p.S) return p.cache_base + p.prox0[h] + (size_t)key * D;
    if (key < p.n - p.W) return p.cache_base + p.dist0[h] + (size_t)(key - p.S) * D;
    return p.cache_base + p.prox0[h] + (size_t)(p.S + (key - p.S) % p.W) * D;
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

// Query rows in LDS: a chunk of kSelChunkRows rows (8 blocks of 32) of one kv head, row-major, rows padded by 16
// bytes so that the 16 lanes of one LDS access (rows r .. r + 15, same column) fall into different banks.  A
// workgroup stages a chunk once and every fragment it then needs comes out of LDS: the keys are read from global
// memory once per workgroup and chunk instead of once per MFMA.
constexpr int kSelChunkBlocks = 8;
constexpr int kSelChunkRows = 32 * kSelChunkBlocks;
template <int D> constexpr int kSelRowBytes = D * 2 + 16;

template <int D>
__device__ inline void stage_query_rows(const select_params &p, int h, int row0, char *lds)
{
    constexpr int cpr = D / 8; // 16-byte pieces per row
    for (int idx = threadIdx.x; idx < kSelChunkRows * cpr; idx += kSelThreads) {
        const int row = idx / cpr, c = idx % cpr;
        sel_u32x4 val = {0, 0, 0, 0}; // rows past the end: zeros (their logits are never used)
        if (row0 + row < p.R) val = *(const sel_u32x4 *)(query_row(p, h, row0 + row, D) + c * 8);
        *(sel_u32x4 *)(lds + row * kSelRowBytes<D> + c * 16) = val;
    }
}

template <int D>
__device__ inline void lds_row_fragments(const char *lds, int rb, int lane, sel_u32x4 (&f)[D / 16])
{
    const char *row = lds + (rb * 32 + (lane & 31)) * kSelRowBytes<D> + (lane >> 5) * 16;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) f[kk] = *(const sel_u32x4 *)(row + kk * 32);
}

// First pass.  Workgroup = (piece of keys, kv head, chunk of query rows); a wave walks its key blocks of 32 and, per
// key block, the chunk's row blocks: S^T = K Q^T, a lane owns query row lane % 32 of each row block and keeps that
// row's running maximum and sum of exponentials.
template <int D>
__global__ __launch_bounds__(kSelThreads) void select_stat_kernel(select_params p)
{
    const int h = blockIdx.y;
    if (!((p.head_mask >> h) & 1)) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int key_lo = blockIdx.x * p.keys_per_wg;
    const int key_hi = key_lo + p.keys_per_wg < p.n ? key_lo + p.keys_per_wg : p.n;
    const int row0 = blockIdx.z * kSelChunkRows;
    const int nblk = (p.R - row0 + 31) / 32 < kSelChunkBlocks ? (p.R - row0 + 31) / 32 : kSelChunkBlocks; // row blocks in use
    __shared__ __align__(16) char ldsq[kSelChunkRows * kSelRowBytes<D>];
    __shared__ float2 red[kSelThreads / 64][kSelChunkRows];
    stage_query_rows<D>(p, h, row0, ldsq);
    __syncthreads();
    float m[kSelChunkBlocks], l[kSelChunkBlocks];
    int qpos[kSelChunkBlocks]; // the row's own position: it sees keys 0 .. qpos
#pragma unroll
    for (int rb = 0; rb < kSelChunkBlocks; ++rb) {
        const int r = row0 + rb * 32 + (lane & 31);
        m[rb] = -INFINITY;
        l[rb] = 0.f;
        qpos[rb] = p.n - p.obs + (r < p.R ? r : 0) / p.rep;
    }
    sel_u32x4 kf[D / 16], kn[D / 16];
    auto key_row = [&](int key0) {
        const int key = key0 + (lane & 31) < p.n ? key0 + (lane & 31) : p.n - 1;
        return key_address(p, h, key, D);
    };
    int key0 = key_lo + wave * 32;
    if (key0 < key_hi) load_row_fragments<D>(key_row(key0), lane, kn);
    for (; key0 < key_hi; key0 += kSelKeysPerIter) {
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) kf[kk] = kn[kk];
        if (key0 + kSelKeysPerIter < key_hi) load_row_fragments<D>(key_row(key0 + kSelKeysPerIter), lane, kn); // next block's keys
#pragma unroll
        for (int rb = 0; rb < kSelChunkBlocks; ++rb) {
            if (rb >= nblk) continue; // (the same in every thread)
            sel_u32x4 qf[D / 16];
            lds_row_fragments<D>(ldsq, rb, lane, qf);
            sel_f32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int kk = 0; kk < D / 16; ++kk)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(sel_bf16x8, kf[kk]),
                                                               __builtin_bit_cast(sel_bf16x8, qf[kk]), acc, 0, 0, 0);
            // accumulator e of this lane: key key0 + 8 (e / 4) + 4 (lane / 32) + e % 4, query row lane % 32 of block rb
            float s[16], tmax = -INFINITY;
            if (key0 + 31 <= p.n - p.obs) { // every query of the window sees all 32 keys (whole wave)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    s[e] = acc[e] * p.scale_log2;
                    tmax = fmaxf(tmax, s[e]);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int ke = key0 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                    s[e] = ke <= qpos[rb] ? acc[e] * p.scale_log2 : -INFINITY; // qpos < n: keys past the end drop out too
                    tmax = fmaxf(tmax, s[e]);
                }
            }
            if (tmax > -INFINITY) {
                const float mn = fmaxf(m[rb], tmax);
                float add = 0.f;
#pragma unroll
                for (int e = 0; e < 16; ++e) add += fast_exp2(s[e] - mn);
                l[rb] = l[rb] * exp2f(m[rb] - mn) + add; // m = -inf: l is 0 and stays 0
                m[rb] = mn;
            }
        }
    }
#pragma unroll
    for (int rb = 0; rb < kSelChunkBlocks; ++rb) {
        merge_stat(m[rb], l[rb], __shfl_xor(m[rb], 32), __shfl_xor(l[rb], 32)); // the two lanes of a row hold different keys
        if (lane < 32) red[wave][rb * 32 + lane] = make_float2(m[rb], l[rb]);
    }
    __syncthreads();
    const int r = row0 + threadIdx.x; // kSelThreads == kSelChunkRows: one thread per row of the chunk
    if (r < p.nrb * 32) {
        float M = red[0][threadIdx.x].x, L = red[0][threadIdx.x].y;
        for (int w = 1; w < kSelThreads / 64; ++w) merge_stat(M, L, red[w][threadIdx.x].x, red[w][threadIdx.x].y);
        p.part[((size_t)h * p.npieces + blockIdx.x) * (p.nrb * 32) + r] = make_float2(M, L);
    }
}
static_assert(kSelThreads == kSelChunkRows, "the first pass hands one row of the chunk to every thread");

// one wave per (kv head, query row): lane c holds piece c (at most 64 pieces).  Writes what the second pass
// subtracts from a logit: maximum + log2(sum), so that exp2(logit - that) is the attention weight; +infinity for
// the rows past the end (their weight is then 0).
__global__ __launch_bounds__(kSelThreads) void select_reduce_kernel(select_params p)
{
    const int h = blockIdx.y;
    if (!((p.head_mask >> h) & 1)) return;
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * (kSelThreads / 64) + (threadIdx.x >> 6);
    if (r >= p.nrb * 32) return;
    float m = -INFINITY, l = 0.f;
    if (lane < p.npieces) {
        const float2 t = p.part[((size_t)h * p.npieces + lane) * (p.nrb * 32) + r];
        m = t.x;
        l = t.y;
    }
    float M = m;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
    float L = m > -INFINITY ? l * exp2f(m - M) : 0.f;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) L += __shfl_xor(L, o); // the same order in every lane: all lanes end with the same sum
    if (lane == 0) p.stat[(size_t)h * (p.nrb * 32) + r] = r < p.R && L > 0.f ? M + log2f(L) : INFINITY; // (every row sees key 0: L > 0)
}

// Second pass.  Workgroup = (kSelVoteKeys distant keys, kv head); a wave takes key blocks of 32 and, per key block,
// every chunk's row blocks: S = Q K^T, a lane owns key lane % 32 and adds up the weights of 16 query rows per MFMA
// tile.  A distant key is older than every query of the observation window (obs <= W): no causal test.
constexpr int kSelVoteBlocks = 4;                                  // key blocks per wave
constexpr int kSelVoteKeys = kSelVoteBlocks * kSelKeysPerIter;     // keys per workgroup

template <int D>
__global__ __launch_bounds__(kSelThreads) void select_vote_kernel(select_params p)
{
    const int h = blockIdx.y;
    if (!((p.head_mask >> h) & 1)) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int dist_hi = p.n - p.W;                                         // distant keys: S .. n - W - 1
    const int wg_key0 = p.S + blockIdx.x * kSelVoteKeys;
    __shared__ __align__(16) char ldsq[kSelChunkRows * kSelRowBytes<D>];
    __shared__ __align__(16) float ldsb[kSelChunkRows];
    float vote[kSelVoteBlocks];
#pragma unroll
    for (int kb = 0; kb < kSelVoteBlocks; ++kb) vote[kb] = 0.f;
    for (int row0 = 0; row0 < p.R; row0 += kSelChunkRows) {
        if (row0) __syncthreads(); // everyone is done with the previous chunk
        stage_query_rows<D>(p, h, row0, ldsq);
        {
            const int r = row0 + threadIdx.x; // one row of the chunk per thread
            ldsb[threadIdx.x] = r < p.nrb * 32 ? p.stat[(size_t)h * (p.nrb * 32) + r] : INFINITY;
        }
        __syncthreads();
        const int nblk = (p.R - row0 + 31) / 32 < kSelChunkBlocks ? (p.R - row0 + 31) / 32 : kSelChunkBlocks;
#pragma unroll
        for (int kb = 0; kb < kSelVoteBlocks; ++kb) {
            const int key0 = wg_key0 + (kb * (kSelThreads / 64) + wave) * 32;
            if (key0 >= dist_hi) continue; // (whole wave; no barrier inside)
            const int key = key0 + (lane & 31) < dist_hi ? key0 + (lane & 31) : dist_hi - 1;
            sel_u32x4 kf[D / 16];
            load_row_fragments<D>(key_address(p, h, key, D), lane, kf);
            for (int rb = 0; rb < nblk; ++rb) {
                sel_u32x4 qf[D / 16];
                lds_row_fragments<D>(ldsq, rb, lane, qf);
                sel_f32x16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                for (int kk = 0; kk < D / 16; ++kk)
                    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(sel_bf16x8, qf[kk]),
                                                                   __builtin_bit_cast(sel_bf16x8, kf[kk]), acc, 0, 0, 0);
                // accumulator e of this lane: query row rb * 32 + 8 (e / 4) + 4 (lane / 32) + e % 4 of the chunk, key lane % 32
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    typedef __attribute__((ext_vector_type(4))) float f32x4;
                    const f32x4 bq = *(const f32x4 *)(ldsb + rb * 32 + 8 * e4 + 4 * (lane >> 5));
#pragma unroll
                    for (int j = 0; j < 4; ++j) vote[kb] += fast_exp2(acc[4 * e4 + j] * p.scale_log2 - bq[j]);
                }
            }
        }
    }
#pragma unroll
    for (int kb = 0; kb < kSelVoteBlocks; ++kb) {
        const int key0 = wg_key0 + (kb * (kSelThreads / 64) + wave) * 32;
        const float v = vote[kb] + __shfl_xor(vote[kb], 32); // the two lanes of a key hold different query rows
        if (lane < 32 && key0 + lane < dist_hi) p.votes[(size_t)h * (dist_hi - p.S) + (key0 + lane - p.S)] = v;
    }
}

// order-preserving map of a float's bits to an unsigned (larger float = larger unsigned)
__device__ inline unsigned ordered_bits(float x)
{
    unsigned u = __builtin_bit_cast(unsigned, x);
    if (u == 0x80000000u) u = 0u; // -0 and +0 are one value
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Selection, one workgroup per kv head, over the pooled votes: find the keep-th largest by four rounds of 8-bit
// histograms over the ordered bit patterns, then write the indices of the selected tokens in ascending order
// (everything above the threshold, and the first `need` of those equal to it).  A thread owns a run of
// ceil(m / 1024) consecutive tokens and keeps the first kTopCache of them in registers, so the five passes read
// memory only for prompts of more than 1024 * kTopCache distant tokens; token order is thread order, so one scan
// over the threads' counts gives every thread the place of its first selected token.
constexpr int kTopCache = 32;

__device__ inline float pooled_vote(const float *__restrict__ v, int t, int m, int r, int width, int use_max)
{
    const int lo = t - r > 0 ? t - r : 0, hi = t + r + 1 < m ? t + r + 1 : m;
    if (use_max) {
        float x = v[lo];
        for (int u = lo + 1; u < hi; ++u) x = fmaxf(x, v[u]);
        return x;
    }
    float acc = 0.f;
    for (int u = lo; u < hi; ++u) acc = acc + v[u];
    return acc / (float)width;
}

// pooling: one thread per (kv head, distant token), so that the window's loads of many tokens are in flight together
// (a thread of select_top_kernel walking its own run would wait for them one after the other)
__global__ __launch_bounds__(256) void select_pool_kernel(const float *__restrict__ votes, int m, uint64_t head_mask, int width,
                                                          int use_max, float *__restrict__ pooled)
{
    const int h = blockIdx.y, t = blockIdx.x * 256 + threadIdx.x;
    if (!((head_mask >> h) & 1) || t >= m) return;
    pooled[(size_t)h * m + t] = pooled_vote(votes + (size_t)h * m, t, m, width / 2, width, use_max);
}

__global__ __launch_bounds__(kTopThreads) void select_top_kernel(const float *__restrict__ pooled, int m, uint64_t head_mask, int keep,
                                                                 int32_t *sel, int sel_stride)
{
    const int h = blockIdx.x;
    if (!((head_mask >> h) & 1)) return;
    const float *pl = pooled + (size_t)h * m;
    int32_t *out = sel + (size_t)h * sel_stride;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int span = (m + kTopThreads - 1) / kTopThreads; // tokens per thread: t0 .. t0 + span - 1 (those below m)
    const int t0 = tid * span;
    unsigned ck[kTopCache]; // ordered bit patterns of the pooled votes of tokens t0 + j
#pragma unroll
    for (int j = 0; j < kTopCache; ++j) { // (loads of clamped addresses, all in flight; what is not this thread's is zeroed after)
        const int t = t0 + j < m ? t0 + j : m - 1;
        ck[j] = ordered_bits(pl[t]);
    }
#pragma unroll
    for (int j = 0; j < kTopCache; ++j)
        if (!(j < span && t0 + j < m)) ck[j] = 0u;
    __shared__ unsigned hist[256];
    __shared__ unsigned s_prefix, s_need;
    __shared__ unsigned wave_tot[2][kTopThreads / 64];
    if (tid == 0) { s_prefix = 0; s_need = (unsigned)keep; }
    __syncthreads();
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        const unsigned prefix = s_prefix, need_in = s_need;
        // The first round's digit is the sign and most of the exponent: pooled votes share a handful of values, and
        // one LDS atomic per token would queue up on those few counters, so there a wave adds each distinct digit once.
        auto count = [&](unsigned key, bool valid) {
            const unsigned digit = (key >> shift) & 255u;
            if (shift == 24) {
                unsigned long long todo = __ballot(valid);
                while (todo) {
                    const int leader = __ffsll((long long)todo) - 1;
                    const unsigned d = (unsigned)__builtin_amdgcn_readlane((int)digit, leader); // (leader is the same in every lane)
                    const unsigned long long same = __ballot(valid && digit == d);
                    if (lane == leader) atomicAdd(&hist[d], (unsigned)__popcll(same));
                    todo &= ~same;
                }
            } else if (valid && (key >> (shift + 8)) == (prefix >> (shift + 8))) {
                atomicAdd(&hist[digit], 1u);
            }
        };
#pragma unroll
        for (int j = 0; j < kTopCache; ++j)
            if (j < span) count(ck[j], t0 + j < m); // (the same test in every thread)
        for (int j = kTopCache; j < span; ++j) count(t0 + j < m ? ordered_bits(pl[t0 + j]) : 0u, t0 + j < m);
        __syncthreads();
        // thread d < 256: candidates with digit >= d (suffix sums by wave, then over the waves above); the digit whose
        // bucket holds the need-th largest candidate is the one with fewer than `need` above it and at least `need` from it on
        unsigned mine = 0, from_here = 0;
        if (tid < 256) {
            mine = hist[tid];
            from_here = mine;
            for (int o = 1; o < 64; o <<= 1) {
                const unsigned up = __shfl_down(from_here, o);
                if (lane + o < 64) from_here += up;
            }
            if (lane == 0) wave_tot[0][wave] = from_here;
        }
        __syncthreads();
        if (tid < 256) {
            for (int w = wave + 1; w < 4; ++w) from_here += wave_tot[0][w];
            const unsigned above = from_here - mine;
            if (above < need_in && need_in <= from_here) {
                s_prefix = prefix | ((unsigned)tid << shift);
                s_need = need_in - above;
            }
        }
        __syncthreads();
    }
    const unsigned thr = s_prefix, need = s_need; // need >= 1 entries equal to the threshold are taken, earliest first
    // tokens above / at the threshold in this thread's run, then in all runs before it
    unsigned n_gt = 0, n_eq = 0;
#pragma unroll
    for (int j = 0; j < kTopCache; ++j)
        if (j < span && t0 + j < m) { n_gt += ck[j] > thr; n_eq += ck[j] == thr; }
    for (int j = kTopCache; j < span; ++j)
        if (t0 + j < m) { const unsigned key = ordered_bits(pl[t0 + j]); n_gt += key > thr; n_eq += key == thr; }
    unsigned inc_gt = n_gt, inc_eq = n_eq;
    for (int o = 1; o < 64; o <<= 1) {
        const unsigned a = __shfl_up(inc_gt, o), b = __shfl_up(inc_eq, o);
        if (lane >= o) { inc_gt += a; inc_eq += b; }
    }
    if (lane == 63) { wave_tot[0][wave] = inc_gt; wave_tot[1][wave] = inc_eq; }
    __syncthreads();
    unsigned gt_before = inc_gt - n_gt, eq_before = inc_eq - n_eq;
    for (int w = 0; w < wave; ++w) { gt_before += wave_tot[0][w]; eq_before += wave_tot[1][w]; }
    auto place = [&](int t, unsigned key) {
        const bool gt = key > thr, eq = key == thr;
        if (gt || (eq && eq_before < need)) {
            const unsigned pos = gt_before + (eq_before < need ? eq_before : need);
            if (pos < (unsigned)keep) out[pos] = t;
        }
        gt_before += gt;
        eq_before += eq;
    };
#pragma unroll
    for (int j = 0; j < kTopCache; ++j)
        if (j < span && t0 + j < m) place(t0 + j, ck[j]);
    for (int j = kTopCache; j < span; ++j)
        if (t0 + j < m) place(t0 + j, ordered_bits(pl[t0 + j]));
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

int pod_launch_select_votes(const pod_cache *c, int layer, int b, uint64_t head_mask, int n, const void *q_obs, int obs, const void *k,
                            float scale, float *votes, void *ws, hipStream_t st)
{
    const pod_layout &ly = c->ly;
    const select_plan s = plan_votes(ly, n, obs);
    select_params p;
    p.q_obs = (const pod_bf16 *)q_obs; p.k = (const pod_bf16 *)k;
    p.cache_base = (const pod_bf16 *)c->base;
    const pod_headmap hm = pod_make_headmap(c, layer);
    for (int h = 0; h < ly.Hkv; ++h) {
        p.prox0[h] = ly.off_proxK / 2 + pod_prox_row0(ly, layer, b, h) * (size_t)ly.D;
        p.dist0[h] = ly.off_distK / 2 + pod_distk_row0(ly, hm, b, h) * (size_t)ly.D;
    }
    p.n = n; p.obs = obs; p.Hq = ly.Hq; p.Hkv = ly.Hkv; p.rep = ly.rep; p.S = ly.S; p.W = ly.W;
    p.R = s.R; p.nrb = s.nrb; p.keys_per_wg = s.keys_per_wg; p.npieces = s.npieces;
    p.scale_log2 = scale * kLog2e;
    p.head_mask = head_mask;
    p.part = (float2 *)ws; p.stat = (float *)((char *)ws + s.off_stat); p.votes = votes;
    const int n_dist = n - ly.S - ly.W;
    const dim3 g1(s.npieces, ly.Hkv, (s.R + kSelChunkRows - 1) / kSelChunkRows), g2((s.nrb * 32 + kSelThreads / 64 - 1) / (kSelThreads / 64), ly.Hkv), g3((n_dist + kSelVoteKeys - 1) / kSelVoteKeys, ly.Hkv);
    if (ly.D == 128) {
        hipLaunchKernelGGL(select_stat_kernel<128>, g1, dim3(kSelThreads), 0, st, p);
        hipLaunchKernelGGL(select_reduce_kernel, g2, dim3(kSelThreads), 0, st, p);
        hipLaunchKernelGGL(select_vote_kernel<128>, g3, dim3(kSelThreads), 0, st, p);
    } else {
        hipLaunchKernelGGL(select_stat_kernel<64>, g1, dim3(kSelThreads), 0, st, p);
        hipLaunchKernelGGL(select_reduce_kernel, g2, dim3(kSelThreads), 0, st, p);
        hipLaunchKernelGGL(select_vote_kernel<64>, g3, dim3(kSelThreads), 0, st, p);
    }
    POD_HIP_TRY(hipGetLastError());
    return POD_OK;
}

int pod_launch_select_top(int Hkv, uint64_t head_mask, const float *votes, int m, int width, int use_max, int keep,
                          float *pooled, int32_t *sel, int sel_stride, hipStream_t st)
{
    hipLaunchKernelGGL(select_pool_kernel, dim3((m + 255) / 256, Hkv), dim3(256), 0, st, votes, m, head_mask, width, use_max, pooled);
    hipLaunchKernelGGL(select_top_kernel, dim3(Hkv), dim3(kTopThreads), 0, st, (const float *)pooled, m, head_mask, keep, sel, sel_stride);
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
