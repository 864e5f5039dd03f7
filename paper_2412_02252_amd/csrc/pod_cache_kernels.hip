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
