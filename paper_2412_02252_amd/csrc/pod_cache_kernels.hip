// Cache maintenance kernels: header clear, append with demotion, prompt fill, logical export.
// Pure index arithmetic and 16-byte copies of bf16 rows: results are bit-exact by construction.
//
// Region rule (derived from the index ranges of Eq. 3 of the paper): with n tokens stored,
// positions [0,S) are sink tokens, the last min(W, n-S) positions are the recent window and
// everything between is distant.  Distant keys are kept only by the lowest layer of a block.
#include "pod_internal.h"

namespace {

constexpr int kThreads = 256;

__device__ inline int32_t *lens_ptr(char *base, const pod_layout &ly) { return (int32_t *)(base + ly.off_lens); }
__device__ inline int32_t *flag_ptr(char *base, const pod_layout &ly) { return (int32_t *)(base + ly.off_flag); }

__global__ void clear_header_kernel(char *base, pod_layout ly, int seq_slot)
{
    const int total = ly.L * ly.B;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x)
        if (seq_slot < 0 || i % ly.B == seq_slot) lens_ptr(base, ly)[i] = 0;
    if (seq_slot < 0 && blockIdx.x == 0 && threadIdx.x == 0) *flag_ptr(base, ly) = 0;
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
