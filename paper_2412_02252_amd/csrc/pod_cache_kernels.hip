// Cache maintenance kernels: header clear, append with demotion, prompt fill, logical export.
// Pure index arithmetic and 16-byte copies of bf16 rows: results are bit-exact by construction.
//
// Region rule (derived from the index ranges of Eq. 3 of the paper): with n tokens stored,
// positions [0,S) are sink tokens, the last min(W, n-S) positions are the recent window and
// everything between is distant.  Distant keys are kept only by the lowest layer of a block.
#include "pod_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kCountsPerLaunch = 256; // sequences one append_many launch covers (their counts travel as kernel arguments)

__device__ inline int32_t *lens_ptr(char *base, const pod_layout &ly) { return (int32_t *)(base + ly.off_lens); }
__device__ inline int32_t *flag_ptr(char *base, const pod_layout &ly) { return (int32_t *)(base + ly.off_flag); }

__global__ void clear_header_kernel(char *base, pod_layout ly, int seq_slot)
{
    const int total = ly.L * ly.B;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x)
        if (seq_slot < 0 || i % ly.B == seq_slot) lens_ptr(base, ly)[i] = 0;
    if (seq_slot < 0 && blockIdx.x == 0 && threadIdx.x == 0) *flag_ptr(base, ly) = 0;
    // arrival counters of the decode kernels (zero whenever no decode kernel is running)
    unsigned long long *tickets = (unsigned long long *)(base + ly.off_tickets);
    int32_t *done = (int32_t *)(base + ly.off_stepdone);
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < ly.B * ly.Hkv; i += gridDim.x * blockDim.x)
        if (seq_slot < 0 || i / ly.Hkv == seq_slot) tickets[i] = 0;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < ly.B; i += gridDim.x * blockDim.x)
        if (seq_slot < 0 || i == seq_slot) done[i] = 0;
}

// One block per sequence.  Each thread moves 16-byte pieces of the (kv head, dim) row.
__global__ void append_kernel(char *base, pod_layout ly, pod_headmap hm, int layer, const uint4 *__restrict__ k_new,
                              const uint4 *__restrict__ v_new, const int32_t *__restrict__ positions)
{
    const int b = blockIdx.x;
    int32_t *lens = lens_ptr(base, ly) + (size_t)layer * ly.B + b;
    const int cpr = ly.D / 8; // 16-byte pieces per head row
    const int pieces = ly.Hkv * cpr;
    // The new rows do not depend on the position check: their loads go out with it.
    const size_t src0 = (size_t)b * pieces + (threadIdx.x < pieces ? threadIdx.x : 0);
    uint4 kn = k_new[src0], vn = v_new[src0];
    const int p = positions[b];
    const int cur = *lens;
    if (p != cur || p < 0 || p >= ly.maxctx) { // uniform over the block
        if (threadIdx.x == 0) atomicOr(flag_ptr(base, ly), 1);
        return;
    }
    const int slot = p < ly.S ? p : ly.S + (p - ly.S) % ly.W;
    const bool demote = p >= ly.P;          // the ring slot holds position p - W
    uint4 *proxK = (uint4 *)(base + ly.off_proxK);
    uint4 *proxV = (uint4 *)(base + ly.off_proxV);
    uint4 *distK = (uint4 *)(base + ly.off_distK);
    uint4 *distV = (uint4 *)(base + ly.off_distV);
    for (int idx = threadIdx.x; idx < pieces; idx += blockDim.x) {
        const int h = idx / cpr, c = idx % cpr;
        const size_t pr = (pod_prox_row0(ly, layer, b, h) + slot) * cpr + c;
        if (idx != (int)threadIdx.x) {
            kn = k_new[(size_t)b * pieces + idx];
            vn = v_new[(size_t)b * pieces + idx];
        }
        if (demote) {
            const size_t t = (size_t)(p - ly.P); // distant row of position p - W
            distV[(pod_dist_row0(ly, layer, b, h) + t) * cpr + c] = proxV[pr];
            if ((hm.lowest_mask >> h) & 1) distK[(pod_distk_row0(ly, hm, b, h) + t) * cpr + c] = proxK[pr];
        }
        proxK[pr] = kn;
        proxV[pr] = vn;
    }
    __syncthreads(); // every thread has read *lens (through cur) before it changes
    if (threadIdx.x == 0) *lens = p + 1;
}

// Several tokens per sequence in one launch: the state after the call is the state after appending
// them one at a time.  blockIdx.y = sequence, grid-stride over 16-byte pieces of its new rows
// [cnt][Hkv][D].  With n0 tokens stored and n1 = n0 + cnt afterwards, new position p goes to
//   its sink slot                          if p < S,
//   distant row p - S directly             if p < n1 - W   (it has left the window by the end of the call),
//   ring slot S + (p - S) % W              otherwise; what that slot held (the last stored position below n0
//                                          that maps to it, if any) is first moved to its distant row.
// The positions of the last case are fewer than W + 1 consecutive ones, so each ring slot is touched by one
// thread per piece: no ordering between threads is needed.  The lengths are left alone (every workgroup
// reads them); commit_lens_kernel stores the new ones afterwards.
struct pod_counts { int32_t cnt[kCountsPerLaunch]; };

__global__ void append_many_kernel(char *base, pod_layout ly, pod_headmap hm, int layer, int b_first, int b0, int T, pod_counts counts,
                                   const uint4 *__restrict__ k_new, const uint4 *__restrict__ v_new,
                                   const int32_t *__restrict__ positions)
{
    const int b = b0 + blockIdx.y;
    const int cnt = counts.cnt[blockIdx.y];
    if (cnt <= 0) return;
    const int n0 = lens_ptr(base, ly)[(size_t)layer * ly.B + b];
    if ((positions && positions[b] != n0) || n0 < 0 || n0 + cnt > ly.maxctx) return; // commit_lens_kernel raises the flag
    const int n1 = n0 + cnt;
    const int cpr = ly.D / 8;
    uint4 *proxK = (uint4 *)(base + ly.off_proxK);
    uint4 *proxV = (uint4 *)(base + ly.off_proxV);
    uint4 *distK = (uint4 *)(base + ly.off_distK);
    uint4 *distV = (uint4 *)(base + ly.off_distV);
    const size_t total = (size_t)cnt * ly.Hkv * cpr;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
        const int c = (int)(idx % cpr);
        const int h = (int)((idx / cpr) % ly.Hkv);
        const int t = (int)(idx / ((size_t)cpr * ly.Hkv));
        const int p = n0 + t;
        const size_t src = ((size_t)(b - b_first) * T + t) * ly.Hkv * cpr + (size_t)h * cpr + c; // rows start at sequence b_first
        const uint4 kn = k_new[src], vn = v_new[src];
        const bool low = (hm.lowest_mask >> h) & 1;
        if (p >= ly.S && p < n1 - ly.W) {
            const size_t r = (size_t)(p - ly.S);
            distV[(pod_dist_row0(ly, layer, b, h) + r) * cpr + c] = vn;
            if (low) distK[(pod_distk_row0(ly, hm, b, h) + r) * cpr + c] = kn;
            continue;
        }
        const int slot = p < ly.S ? p : ly.S + (p - ly.S) % ly.W;
        const size_t pr = (pod_prox_row0(ly, layer, b, h) + slot) * cpr + c;
        if (p >= ly.S) {
            const int held = p - ((p - n0) / ly.W + 1) * ly.W; // the stored position in this ring slot
            if (held >= ly.S) {
                const size_t r = (size_t)(held - ly.S);
                distV[(pod_dist_row0(ly, layer, b, h) + r) * cpr + c] = proxV[pr];
                if (low) distK[(pod_distk_row0(ly, hm, b, h) + r) * cpr + c] = proxK[pr];
            }
        }
        proxK[pr] = kn;
        proxV[pr] = vn;
    }
}

// One thread per sequence of the launch above: store the new length, or raise the flag if the
// start position was not the stored length.
__global__ void commit_lens_kernel(char *base, pod_layout ly, int layer, int b0, int nb, pod_counts counts,
                                   const int32_t *__restrict__ positions)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nb || counts.cnt[i] <= 0) return;
    int32_t *len = lens_ptr(base, ly) + (size_t)layer * ly.B + b0 + i;
    const int n0 = *len;
    if ((positions && positions[b0 + i] != n0) || n0 < 0 || n0 + counts.cnt[i] > ly.maxctx) atomicOr(flag_ptr(base, ly), 1);
    else *len = n0 + counts.cnt[i];
}

// Contiguous K/V [n][Hkv][D] of one sequence for the chunk attention: positions below p0 (the stored
// length) come out of the cache, positions p0 .. p0 + T - 1 from the chunk's own rows.
//   v_all : this layer's values (every position is stored)
//   k_all : this layer's keys where it keeps them (sink, recent window, and distant positions of the heads
//           for which the layer is the lowest of the block); zeros elsewhere (never counted by Eq. 3 for a
//           query at or after p0)
//   ks_all: for the other heads, the keys of the lowest layer of the head's block, wherever that layer holds
//           them at ITS current length (it may have stored the chunk already); heads that are lowest here
//           are skipped
struct pod_gather_args {
    int32_t low_layer[kMaxKvHeads]; // lowest layer of head h's block
    int32_t low_row[kMaxKvHeads];   // slot * B of the distant-key store of that block
};

__global__ void gather_kernel(const char *base, pod_layout ly, pod_gather_args ga, uint64_t lowest_mask, int layer, int b,
                              int p0, int T, const uint4 *__restrict__ k_chunk, const uint4 *__restrict__ v_chunk,
                              const uint4 *__restrict__ ks_chunk, uint4 *k_all, uint4 *v_all, uint4 *ks_all)
{
    // blockIdx.y = kv head: everything that depends on the head is uniform over the block, and the index
    // arithmetic per piece is a shift and a mask (D / 8 is 8 or 16)
    const int h = blockIdx.y;
    const int cpr = ly.D / 8, cshift = ly.D == 128 ? 4 : 3;
    const uint4 *proxK = (const uint4 *)(base + ly.off_proxK);
    const uint4 *proxV = (const uint4 *)(base + ly.off_proxV);
    const uint4 *distK = (const uint4 *)(base + ly.off_distK);
    const uint4 *distV = (const uint4 *)(base + ly.off_distV);
    const int32_t *lens = (const int32_t *)(base + ly.off_lens);
    const int rec_lo = p0 - ly.W > ly.S ? p0 - ly.W : ly.S;   // first position of this layer's recent window
    const bool low = (lowest_mask >> h) & 1;
    const bool want_ks = !low && ks_all;
    const int la = ga.low_layer[h];
    const int na = want_ks ? lens[(size_t)la * ly.B + b] : 0;  // p0, or p0 + T if that layer took the chunk already
    const int rec_a = na - ly.W > ly.S ? na - ly.W : ly.S;
    const size_t own_prox = pod_prox_row0(ly, layer, b, h), low_prox = pod_prox_row0(ly, la, b, h);
    const size_t own_dist = pod_dist_row0(ly, layer, b, h), key_dist = (size_t)(ga.low_row[h] + b) * ly.Cd;
    const size_t total = (size_t)(p0 + T) << cshift;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
        const int c = (int)(idx & (cpr - 1));
        const int j = (int)(idx >> cshift);
        const size_t dst = (((size_t)j * ly.Hkv + h) << cshift) + c;
        if (j >= p0) {
            const size_t src = (((size_t)(j - p0) * ly.Hkv + h) << cshift) + c;
            k_all[dst] = k_chunk[src];
            v_all[dst] = v_chunk[src];
            if (want_ks) ks_all[dst] = ks_chunk[src];
            continue;
        }
        const int slot = j < ly.S ? j : ly.S + (j - ly.S) % ly.W;
        const size_t r = (size_t)(j - ly.S);
        uint4 kk = make_uint4(0, 0, 0, 0), vv;
        if (j < ly.S || j >= rec_lo) {
            kk = proxK[((own_prox + slot) << cshift) + c];
            vv = proxV[((own_prox + slot) << cshift) + c];
        } else {
            vv = distV[((own_dist + r) << cshift) + c];
            if (low) kk = distK[((key_dist + r) << cshift) + c];
        }
        k_all[dst] = kk;
        v_all[dst] = vv;
        if (want_ks)
            ks_all[dst] = (j < ly.S || j >= rec_a) ? proxK[((low_prox + slot) << cshift) + c] : distK[((key_dist + r) << cshift) + c];
    }
}

// ---------------------------------------------------------------------------------------------
// Chunk attention without a contiguous copy of the sequence.
//
// chunk_update_kernel stores the chunk first (the state afterwards is pod_cache_append_many's).  Every key and
// value the chunk's queries need then lies in the cache at its new length n = p0 + T, with one exception: a head
// whose block has a lower layer drops its own keys when they leave the recent window, and the chunk's queries
// still need those that are inside the window at the QUERY's position (Eq. 3 with the window taken there).  So
// the update keeps the keys it drops, positions max(S, p0 - W) .. n - W - 1, in the caller's workspace (the
// "spill", [Hkv][rows][D]).  Seen from one kv head, position j of a stream (0 = this layer's keys, 1 = its values,
// 2 = the keys of the lowest layer of the head's block) is then a row of one of a few runs of consecutive rows,
// all with rows D * 2 bytes apart:
//   sink slots [0, S) | distant store, or nothing, then the spill [S, rec_lo) | ring up to its wrap | ring after it
// with rec_lo = max(S, n - W).  The attention kernel requests whole tiles of 64 positions by ONE address.  The
// update launch also writes that address for every (stream, head, tile): the tile's first row where the whole
// tile lies in one run, else a staging slot that chunk_dirty_kernel fills afterwards with the tile's rows one by
// one.  The runs change at four positions at most (S, the spill's first position, rec_lo, the wrap), hence
// four staging slots per stream and head, slot i for the tile that holds boundary i in its inside (a tile with
// several takes the first).
constexpr int kChunkTile = 64;
constexpr int kChunkSlots = 4;
struct chunk_view {
    pod_layout ly;
    pod_gather_args ga;
    uint64_t lowest_mask;
    int layer, b, p0, n;
    int first_spill; // max(S, p0 - W)
    int rec_lo;      // first position the ring holds at length n
    int wrap;        // first position stored after the ring's wrap (>= n: the ring does not wrap)
    int spill_rows;  // rows per head in the spill
    int ntiles;
    unsigned long long *tab; // [3][Hkv][ntiles]
    char *spill, *dirty;     // dirty: [3][Hkv][kChunkSlots][kChunkTile][D]
};
enum { kRunSink, kRunNone, kRunStore, kRunRingA, kRunRingB };
struct chunk_row { int run; const char *ptr; };

__device__ inline chunk_row chunk_src(const char *base, const chunk_view &cv, int stream, int h, int j)
{
    const pod_layout &ly = cv.ly;
    const size_t rb = (size_t)ly.D * 2;
    const int lay = stream == 2 ? cv.ga.low_layer[h] : cv.layer;
    const char *prox = base + (stream == 1 ? ly.off_proxV : ly.off_proxK) + pod_prox_row0(ly, lay, cv.b, h) * rb;
    if (j < ly.S) return {kRunSink, prox + (size_t)j * rb};
    if (j >= cv.rec_lo) {
        if (j < cv.wrap) return {kRunRingA, prox + (size_t)(ly.S + (cv.rec_lo - ly.S) % ly.W + (j - cv.rec_lo)) * rb};
        return {kRunRingB, prox + (size_t)(ly.S + (j - cv.wrap)) * rb};
    }
    const size_t r = (size_t)(j - ly.S);
    if (stream == 1) return {kRunStore, base + ly.off_distV + (pod_dist_row0(ly, cv.layer, cv.b, h) + r) * rb};
    if (stream == 2 || ((cv.lowest_mask >> h) & 1))
        return {kRunStore, base + ly.off_distK + ((size_t)(cv.ga.low_row[h] + cv.b) * ly.Cd + r) * rb};
    if (j >= cv.first_spill) return {kRunStore, cv.spill + ((size_t)h * cv.spill_rows + (j - cv.first_spill)) * rb};
    return {kRunNone, nullptr}; // a key this layer dropped before the chunk: outside every window of the chunk's queries
}

// index of the first run boundary strictly inside positions (j0, jl], or -1
__device__ inline int chunk_first_boundary(const chunk_view &cv, int j0, int jl)
{
    const int bv[kChunkSlots] = {cv.ly.S, cv.first_spill, cv.rec_lo, cv.wrap};
#pragma unroll
    for (int i = 0; i < kChunkSlots; ++i)
        if (bv[i] > j0 && bv[i] <= jl) return i;
    return -1;
}

__device__ inline char *chunk_dirty_slot(const chunk_view &cv, int stream, int h, int i)
{
    return cv.dirty + ((((size_t)stream * cv.ly.Hkv + h) * kChunkSlots + i) * kChunkTile) * ((size_t)cv.ly.D * 2);
}

// blockIdx.y = kv head.  Grid-stride over the 16-byte pieces of the head's T new rows, then over its table entries.
__global__ void chunk_update_kernel(char *base, chunk_view cv, int T, const uint4 *__restrict__ k_new,
                                    const uint4 *__restrict__ v_new)
{
    const pod_layout &ly = cv.ly;
    const int h = blockIdx.y, b = cv.b, layer = cv.layer;
    const int32_t *len = lens_ptr(base, ly) + (size_t)layer * ly.B + b;
    const int n0 = cv.p0, n1 = cv.n;
    {
        const int cpr = ly.D / 8, cshift = ly.D == 128 ? 4 : 3;
        uint4 *proxK = (uint4 *)(base + ly.off_proxK);
        uint4 *proxV = (uint4 *)(base + ly.off_proxV);
        uint4 *distK = (uint4 *)(base + ly.off_distK);
        uint4 *distV = (uint4 *)(base + ly.off_distV);
        const bool low = (cv.lowest_mask >> h) & 1;
        const size_t own_prox = pod_prox_row0(ly, layer, b, h), own_dist = pod_dist_row0(ly, layer, b, h);
        const size_t key_dist = (size_t)(cv.ga.low_row[h] + b) * ly.Cd;
        uint4 *spill = (uint4 *)cv.spill + (((size_t)h * cv.spill_rows) << cshift);
        // where the key of distant position j goes: the block's store (lowest layer), or the spill for this call
        auto keep_key = [&](int j, int c, uint4 kk) {
            if (low) distK[((key_dist + (size_t)(j - ly.S)) << cshift) + c] = kk;
            else spill[((size_t)(j - cv.first_spill) << cshift) + c] = kk;
        };
        // Every address below follows from the launch arguments, so the loads of a piece (its new rows and what its
        // ring slot holds) go out together with the load of the stored length; nothing is stored before that test.
        const int stored = *len;
        const bool ok = stored == n0 && n0 >= 0 && n1 <= ly.maxctx;
        const size_t total = (size_t)T << cshift;
        for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
            const int c = (int)(idx & (cpr - 1));
            const int t = (int)(idx >> cshift);
            const int p = n0 + t;
            const size_t src = (((size_t)t * ly.Hkv + h) << cshift) + c;
            const uint4 kn = k_new[src], vn = v_new[src];
            const bool straight = p >= ly.S && p < n1 - ly.W; // has left the window by the end of the call
            const int slot = p < ly.S ? p : ly.S + (p - ly.S) % ly.W;
            const size_t pr = ((own_prox + slot) << cshift) + c;
            const int held = p - ((p - n0) / ly.W + 1) * ly.W;      // the stored position in this ring slot
            const bool moves = !straight && p >= ly.S && held >= ly.S;
            uint4 ko = make_uint4(0, 0, 0, 0), vo = ko;
            if (moves) { ko = proxK[pr]; vo = proxV[pr]; }
            if (!ok) break;
            if (straight) {
                distV[((own_dist + (size_t)(p - ly.S)) << cshift) + c] = vn;
                keep_key(p, c, kn);
                continue;
            }
            if (moves) {
                distV[((own_dist + (size_t)(held - ly.S)) << cshift) + c] = vo;
                keep_key(held, c, ko);
            }
            proxK[pr] = kn;
            proxV[pr] = vn;
        }
        // tile addresses of this head, as they hold once every workgroup of this launch is done.  They follow from the
        // launch arguments alone and are written whatever the length test said: the attention launch then reads
        // valid memory in any case (and raises the flag after the same test).
        const int entries = 3 * cv.ntiles;
        for (int e = blockIdx.x * blockDim.x + threadIdx.x; e < entries; e += gridDim.x * blockDim.x) {
            const int stream = e / cv.ntiles, kt = e - stream * cv.ntiles;
            const int j0 = kt * kChunkTile, jl = min(j0 + kChunkTile, n1) - 1;
            const chunk_row first = chunk_src(base, cv, stream, h, j0), last = chunk_src(base, cv, stream, h, jl);
            const char *a;
            if (first.run == last.run) a = first.run == kRunNone ? chunk_dirty_slot(cv, stream, h, 0) : first.ptr; // (never requested: any valid rows)
            else a = chunk_dirty_slot(cv, stream, h, max(chunk_first_boundary(cv, j0, jl), 0));
            cv.tab[((size_t)stream * ly.Hkv + h) * cv.ntiles + kt] = (unsigned long long)a;
        }
    }
    // (the length is not stored here: every workgroup tests it.  The attention launch that follows stores it.)
}

// blockIdx.x = stream * kChunkSlots + boundary, blockIdx.y = kv head: copies the rows of the tile that has this
// boundary inside into its staging slot (zeros where the stream holds nothing).  Runs after chunk_update_kernel.
__global__ void chunk_dirty_kernel(const char *base, chunk_view cv)
{
    const pod_layout &ly = cv.ly;
    const int i = blockIdx.x % kChunkSlots, stream = blockIdx.x / kChunkSlots, h = blockIdx.y;
    const int bv[kChunkSlots] = {ly.S, cv.first_spill, cv.rec_lo, cv.wrap};
    const int v = bv[i];
    if (v <= 0 || v >= cv.n) return;
    const int j0 = v / kChunkTile * kChunkTile, jl = min(j0 + kChunkTile, cv.n) - 1;
    if (chunk_first_boundary(cv, j0, jl) != i) return; // at the tile's first position, or a lower boundary owns the tile
    const int cpr = ly.D / 8;
    uint4 *dst = (uint4 *)chunk_dirty_slot(cv, stream, h, i);
    for (int idx = threadIdx.x; idx < kChunkTile * cpr; idx += blockDim.x) {
        const int r = idx / cpr, c = idx % cpr;
        uint4 val = make_uint4(0, 0, 0, 0);
        if (j0 + r < cv.n) {
            const chunk_row s = chunk_src(base, cv, stream, h, j0 + r);
            if (s.run != kRunNone) val = ((const uint4 *)s.ptr)[c];
        }
        dst[idx] = val;
    }
}

// Grid-stride over 16-byte pieces of the prompt's K/V [n][Hkv][D].
__global__ void fill_kernel(char *base, pod_layout ly, pod_headmap hm, int layer, int b, int n,
                            const uint4 *__restrict__ k, const uint4 *__restrict__ v)
{
    const int cpr = ly.D / 8;
    const int rec_lo = n - ly.W > ly.S ? n - ly.W : ly.S; // first position of the recent window
    uint4 *proxK = (uint4 *)(base + ly.off_proxK);
    uint4 *proxV = (uint4 *)(base + ly.off_proxV);
    uint4 *distK = (uint4 *)(base + ly.off_distK);
    uint4 *distV = (uint4 *)(base + ly.off_distV);
    const size_t total = (size_t)n * ly.Hkv * cpr;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
        const int c = (int)(idx % cpr);
        const int h = (int)((idx / cpr) % ly.Hkv);
        const int p = (int)(idx / ((size_t)cpr * ly.Hkv));
        if (p < ly.S || p >= rec_lo) {
            const int slot = p < ly.S ? p : ly.S + (p - ly.S) % ly.W;
            const size_t pr = (pod_prox_row0(ly, layer, b, h) + slot) * cpr + c;
            proxK[pr] = k[idx];
            proxV[pr] = v[idx];
        } else {
            const size_t t = (size_t)(p - ly.S);
            distV[(pod_dist_row0(ly, layer, b, h) + t) * cpr + c] = v[idx];
            if ((hm.lowest_mask >> h) & 1) distK[(pod_distk_row0(ly, hm, b, h) + t) * cpr + c] = k[idx];
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) lens_ptr(base, ly)[(size_t)layer * ly.B + b] = n;
}

// Gather the logical views [tokens][Hkv][D] in position order.
__global__ void export_kernel(const char *base, pod_layout ly, pod_headmap hm, int layer, int b, int n, uint4 *sinkK,
                              uint4 *sinkV, uint4 *recK, uint4 *recV, uint4 *dK, uint4 *dV)
{
    const int cpr = ly.D / 8;
    const int n_sink = n < ly.S ? n : ly.S;
    const int rec_lo = n - ly.W > ly.S ? n - ly.W : ly.S;
    const uint4 *proxK = (const uint4 *)(base + ly.off_proxK);
    const uint4 *proxV = (const uint4 *)(base + ly.off_proxV);
    const uint4 *distK = (const uint4 *)(base + ly.off_distK);
    const uint4 *distV = (const uint4 *)(base + ly.off_distV);
    const size_t total = (size_t)n * ly.Hkv * cpr;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
        const int c = (int)(idx % cpr);
        const int h = (int)((idx / cpr) % ly.Hkv);
        const int p = (int)(idx / ((size_t)cpr * ly.Hkv));
        if (p < n_sink) {
            const size_t pr = (pod_prox_row0(ly, layer, b, h) + p) * cpr + c;
            const size_t o = ((size_t)p * ly.Hkv + h) * cpr + c;
            if (sinkK) sinkK[o] = proxK[pr];
            if (sinkV) sinkV[o] = proxV[pr];
        } else if (p >= rec_lo) {
            const int slot = ly.S + (p - ly.S) % ly.W;
            const size_t pr = (pod_prox_row0(ly, layer, b, h) + slot) * cpr + c;
            const size_t o = ((size_t)(p - rec_lo) * ly.Hkv + h) * cpr + c;
            if (recK) recK[o] = proxK[pr];
            if (recV) recV[o] = proxV[pr];
        } else {
            const size_t t = (size_t)(p - ly.S);
            const size_t o = (t * ly.Hkv + h) * cpr + c;
            if (dV) dV[o] = distV[(pod_dist_row0(ly, layer, b, h) + t) * cpr + c];
            // (heads for which this layer is not a lowest layer keep no keys here: zeros)
            if (dK) dK[o] = ((hm.lowest_mask >> h) & 1) ? distK[(pod_distk_row0(ly, hm, b, h) + t) * cpr + c] : make_uint4(0, 0, 0, 0);
        }
    }
}

int grid_for(size_t items)
{
    size_t g = (items + kThreads - 1) / kThreads;
    if (g < 1) g = 1;
    if (g > 256 * 32) g = 256 * 32;
    return (int)g;
}

} // namespace

int pod_launch_clear_header(const pod_cache *c, hipStream_t st)
{
    hipLaunchKernelGGL(clear_header_kernel, dim3(grid_for((size_t)c->ly.L * c->ly.B)), dim3(kThreads), 0, st,
                       c->base, c->ly, -1);
    POD_HIP_TRY(hipGetLastError());
    return POD_OK;
}

int pod_launch_reset(const pod_cache *c, int seq_slot, hipStream_t st)
{
    hipLaunchKernelGGL(clear_header_kernel, dim3(grid_for((size_t)c->ly.L * c->ly.B)), dim3(kThreads), 0, st,
                       c->base, c->ly, seq_slot);
    POD_HIP_TRY(hipGetLastError());
    return POD_OK;
}

int pod_launch_append(const pod_cache *c, int layer, const void *k_new, const void *v_new, const int32_t *positions,
                      int B, hipStream_t st)
{
    int threads = c->ly.Hkv * (c->ly.D / 8);
    threads = threads < 64 ? 64 : (threads > 1024 ? 1024 : (threads + 63) / 64 * 64);
    hipLaunchKernelGGL(append_kernel, dim3(B), dim3(threads), 0, st, c->base, c->ly, pod_make_headmap(c, layer), layer, (const uint4 *)k_new,
                       (const uint4 *)v_new, positions);
    POD_HIP_TRY(hipGetLastError());
    return POD_OK;
}

int pod_launch_fill(const pod_cache *c, int layer, int seq_slot, int n, const void *k, const void *v, hipStream_t st)
{
    const size_t items = (size_t)n * c->ly.Hkv * (c->ly.D / 8);
    hipLaunchKernelGGL(fill_kernel, dim3(grid_for(items)), dim3(kThreads), 0, st, c->base, c->ly, pod_make_headmap(c, layer), layer, seq_slot, n,
                       (const uint4 *)k, (const uint4 *)v);
    POD_HIP_TRY(hipGetLastError());
    return POD_OK;
}

int pod_launch_export(const pod_cache *c, int layer, int seq_slot, int64_t n, void *sinkK, void *sinkV, void *recK,
                      void *recV, void *distK, void *distV, hipStream_t st)
{
    const size_t items = (size_t)n * c->ly.Hkv * (c->ly.D / 8);
    hipLaunchKernelGGL(export_kernel, dim3(grid_for(items)), dim3(kThreads), 0, st, (const char *)c->base, c->ly,
                       pod_make_headmap(c, layer), layer, seq_slot, (int)n, (uint4 *)sinkK, (uint4 *)sinkV, (uint4 *)recK, (uint4 *)recV,
                       (uint4 *)distK, (uint4 *)distV);
    POD_HIP_TRY(hipGetLastError());
    return POD_OK;
}

int pod_launch_append_many(const pod_cache *c, int layer, const void *k_new, const void *v_new, const int32_t *positions,
                           const int32_t *counts, int T, int b_first, int B, hipStream_t st)
{
    const pod_headmap hm = pod_make_headmap(c, layer);
    for (int g0 = 0; g0 < B; g0 += kCountsPerLaunch) {
        const int nb = B - g0 < kCountsPerLaunch ? B - g0 : kCountsPerLaunch;
        const int b0 = b_first + g0;
        pod_counts pc;
        int most = 0;
        for (int i = 0; i < kCountsPerLaunch; ++i) {
            pc.cnt[i] = i < nb ? counts[g0 + i] : 0;
            if (pc.cnt[i] > most) most = pc.cnt[i];
        }
        if (most == 0) continue;
        const size_t items = (size_t)most * c->ly.Hkv * (c->ly.D / 8);
        int gx = grid_for(items);
        if (gx > 2048) gx = 2048;
        hipLaunchKernelGGL(append_many_kernel, dim3(gx, nb), dim3(kThreads), 0, st, c->base, c->ly, hm, layer, b_first, b0, T, pc,
                           (const uint4 *)k_new, (const uint4 *)v_new, positions);
        hipLaunchKernelGGL(commit_lens_kernel, dim3((nb + 63) / 64), dim3(64), 0, st, c->base, c->ly, layer, b0, nb, pc, positions);
    }
    POD_HIP_TRY(hipGetLastError());
    return POD_OK;
}

int pod_launch_gather(const pod_cache *c, int layer, int seq_slot, int p0, int T, const void *k_chunk, const void *v_chunk,
                      const void *ks_chunk, void *k_all, void *v_all, void *ks_all, hipStream_t st)
{
    pod_gather_args ga;
    const int H = c->ly.Hkv;
    for (int h = 0; h < kMaxKvHeads; ++h) {
        ga.low_layer[h] = h < H ? c->lowest[(size_t)layer * H + h] : 0;
        ga.low_row[h] = h < H ? c->kslot[(size_t)layer * H + h] * c->ly.B : 0;
    }
    const size_t items = (size_t)(p0 + T) * (c->ly.D / 8);      // per kv head (blockIdx.y)
    int gx = grid_for(items);
    if (gx > 4096 / H + 1) gx = 4096 / H + 1;
    hipLaunchKernelGGL(gather_kernel, dim3(gx, H), dim3(kThreads), 0, st, (const char *)c->base, c->ly, ga,
                       pod_make_headmap(c, layer).lowest_mask, layer, seq_slot, p0, T, (const uint4 *)k_chunk,
                       (const uint4 *)v_chunk, (const uint4 *)ks_chunk, (uint4 *)k_all, (uint4 *)v_all, (uint4 *)ks_all);
    POD_HIP_TRY(hipGetLastError());
    return POD_OK;
}

// workspace of the launches below for a chunk of T tokens that brings the sequence to n_total (T <= 0: any chunk length)
size_t pod_chunk_direct_bytes(const pod_layout &ly, int64_t n_total, int64_t T)
{
    const size_t rb = (size_t)ly.D * 2;
    const size_t ntiles = (size_t)(n_total + kChunkTile - 1) / kChunkTile;
    const size_t tab = (3 * ly.Hkv * ntiles * 8 + 255) / 256 * 256;
    const int64_t rows = T > 0 && T < n_total ? T : n_total; // the update displaces at most as many rows as it stores
    const size_t spill = ((size_t)ly.Hkv * rows * rb + 255) / 256 * 256;
    return tab + spill + (size_t)3 * ly.Hkv * kChunkSlots * kChunkTile * rb;
}

int pod_launch_chunk_update(const pod_cache *c, int layer, int seq_slot, int p0, int T, const void *k_chunk, const void *v_chunk,
                            void *workspace, size_t workspace_bytes, const unsigned long long **tile_tab, int *ntiles,
                            hipStream_t st)
{
    const pod_layout &ly = c->ly;
    const int H = ly.Hkv;
    chunk_view cv;
    cv.ly = ly;
    for (int h = 0; h < kMaxKvHeads; ++h) {
        cv.ga.low_layer[h] = h < H ? c->lowest[(size_t)layer * H + h] : 0;
        cv.ga.low_row[h] = h < H ? c->kslot[(size_t)layer * H + h] * ly.B : 0;
    }
    cv.lowest_mask = pod_make_headmap(c, layer).lowest_mask;
    cv.layer = layer; cv.b = seq_slot; cv.p0 = p0; cv.n = p0 + T;
    cv.first_spill = p0 - ly.W > ly.S ? p0 - ly.W : ly.S;
    cv.rec_lo = cv.n - ly.W > ly.S ? cv.n - ly.W : ly.S;
    cv.wrap = cv.rec_lo + (ly.W - (cv.rec_lo - ly.S) % ly.W);
    cv.spill_rows = cv.rec_lo > cv.first_spill ? cv.rec_lo - cv.first_spill : 0;
    cv.ntiles = (cv.n + kChunkTile - 1) / kChunkTile;
    const size_t rb = (size_t)ly.D * 2;
    const size_t tab_bytes = ((size_t)3 * H * cv.ntiles * 8 + 255) / 256 * 256;
    const size_t spill_bytes = ((size_t)H * cv.spill_rows * rb + 255) / 256 * 256;
    const size_t dirty_bytes = (size_t)3 * H * kChunkSlots * kChunkTile * rb;
    if (workspace_bytes < tab_bytes + spill_bytes + dirty_bytes)
        return pod_fail(POD_ERR_CAPACITY, "chunk workspace too small: %zu < %zu", workspace_bytes, tab_bytes + spill_bytes + dirty_bytes);
    cv.tab = (unsigned long long *)workspace;
    cv.spill = (char *)workspace + tab_bytes;
    cv.dirty = cv.spill + spill_bytes;
    const size_t items = (size_t)T * (ly.D / 8); // per kv head (blockIdx.y)
    int gx = grid_for(items);
    if (gx > 4096 / H + 1) gx = 4096 / H + 1;
    hipLaunchKernelGGL(chunk_update_kernel, dim3(gx, H), dim3(kThreads), 0, st, c->base, cv, T, (const uint4 *)k_chunk,
                       (const uint4 *)v_chunk);
    const int bv[kChunkSlots] = {ly.S, cv.first_spill, cv.rec_lo, cv.wrap};
    bool dirty = false;
    for (int i = 0; i < kChunkSlots; ++i) dirty = dirty || (bv[i] > 0 && bv[i] < cv.n && bv[i] % kChunkTile != 0);
    if (dirty)
        hipLaunchKernelGGL(chunk_dirty_kernel, dim3(3 * kChunkSlots, H), dim3(kThreads), 0, st, (const char *)c->base, cv);
    POD_HIP_TRY(hipGetLastError());
    *tile_tab = cv.tab;
    *ntiles = cv.ntiles;
    return POD_OK;
}
