// Internal declarations shared by the translation units of libpod (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/pod.h"

// ---------------------------------------------------------------------------
// Device-memory layout of one cache.
//
// header   : int32 lens[L][B] (tokens held per layer and slot), int32 flag, arrival counters of the decode kernels
// proxK/V  : [L][B][Hkv][P][D]   P = S + W slots per (layer, slot, kv head):
//            slots [0,S) are the sink tokens, slot S + (p - S) % W is the ring
//            slot of position p >= S.  While fewer than W tokens >= S exist
//            the ring fills from its first slot, so the live proximal rows are
//            always the contiguous slots [0, min(n, P)).
// distV    : [L][B][Hkv][Cd][D]  Cd = max_context - P; row t = position S + t
// distK    : [slots][B][Cd][D]    keys of a block's lowest layer only: one slot per
//            (kv head, block of that head), numbered in (layer, head) order of the lowest
//            layers; uniform blocks of G layers give slot (l / G) * Hkv + h
//
// Head-major on purpose: the rows one (sequence, kv head) pair streams at decode
// time are one contiguous run, so a split-K chunk is a single linear read.
// Offsets are in bytes from the buffer start; every region is 256-byte aligned.
// ---------------------------------------------------------------------------
struct pod_layout {
    int32_t L, G, Hq, Hkv, D, S, W, B, maxctx;
    int32_t P;   // S + W
    int32_t Cd;  // distant rows per (layer, slot, head)
    int32_t rep; // Hq / Hkv
    int32_t nslots; // distant-key stores: (kv head, block) pairs
    size_t off_tickets, off_stepdone; // uint64 [B][Hkv] and int32 [B]: arrival counters of the fused decode kernels (zero between launches)
    size_t off_lens, off_flag, off_proxK, off_proxV, off_distV, off_distK, total_bytes;
};

typedef unsigned short pod_bf16; // raw bits

__host__ __device__ inline size_t pod_prox_row0(const pod_layout &ly, int layer, int b, int h)
{
    return (((size_t)layer * ly.B + b) * ly.Hkv + h) * (size_t)ly.P;
}
__host__ __device__ inline size_t pod_dist_row0(const pod_layout &ly, int layer, int b, int h) // distant values
{
    return (((size_t)layer * ly.B + b) * ly.Hkv + h) * (size_t)ly.Cd;
}

// One layer's view of the block table, passed to kernels by value.
constexpr int kMaxKvHeads = 64;
struct pod_headmap {
    uint64_t lowest_mask;           // bit h: this layer is the lowest of head h's block (it owns that store)
    int32_t uniform_row0;           // >= 0: every head h reads slot row uniform_row0 + h * B (uniform blocks); the
                                    // table below is then not consulted (a per-thread index into kernel arguments
                                    // is a memory load, which the cache-update kernels avoid in the common case)
    int32_t kslot_row[kMaxKvHeads]; // slot * B of the distant-key store head h reads at this layer
};
__host__ __device__ inline size_t pod_distk_row0(const pod_layout &ly, const pod_headmap &hm, int b, int h) // distant keys
{
    const size_t row = hm.uniform_row0 >= 0 ? (size_t)hm.uniform_row0 + (size_t)h * ly.B : (size_t)hm.kslot_row[h];
    return (row + b) * (size_t)ly.Cd;
}

struct pod_cache {
    pod_layout ly;
    char *base;        // device buffer (caller's)
    int64_t *host_len; // [L][B] mirror
    int32_t *lowest;   // [L][Hkv] lowest layer of the block of (layer, kv head)
    int32_t *kslot;    // [L][Hkv] distant-key slot that (layer, kv head) reads
    bool uniform;      // every kv head has the same blocks
    int device;
    // tuning overrides read once from the environment in pod_cache_init (0 = none): tokens per split-K piece of the
    // distant / proximal region (POD_DECODE_CHUNK, POD_DECODE_CHUNK_PROX)
    int tune_chunk, tune_chunk_prox;
    bool fused_merge;      // plain decode merges its partials inside the streaming kernel (POD_DECODE_FUSED=0: separate kernel)
    bool walk_turns;       // the layers of a block walk the block's distant keys in alternating directions (POD_DECODE_WALK_TURNS=0: all forward)
    bool even_split;       // launches of several rounds give every workgroup the same number of rows (POD_DECODE_EVEN=0: fixed pieces)
    bool xcd_local;        // hand partials over inside one XCD's L2 where the launch shape allows (POD_DECODE_XCD_LOCAL=0: never)
    int nxcd;              // XCDs a one-dimensional launch is spread over round-robin (0: no such pattern seen by the probe)
    bool chunk_in_place;   // chunk attention reads keys and values where the cache holds them (POD_CHUNK_IN_PLACE=0: from a contiguous copy)
    bool device_lengths;   // kernels take sequence lengths from the calls' device arrays only (pod_cache_set_length_source)
    // the library's own split-K scratch on `device` (pod_decode_attention_static): device address and size
    void *static_scratch;
    size_t static_scratch_bytes;
    // optional event pairs around the decode partial kernel (pod_profile_*)
    hipEvent_t *prof_ev; // [2 * prof_cap]
    int prof_cap, prof_n;
    void *trace;   // device buffer for per-workgroup clock records of the fused decode launches (pod_profile_set_trace)
    int trace_cap; // workgroups it holds (8 x 8 bytes each)
};

// error reporting (pod_api.hip)
int pod_fail(int code, const char *fmt, ...);
int pod_hip_fail(hipError_t e, const char *what);

#define POD_HIP_TRY(expr)                                        \
    do {                                                         \
        hipError_t e__ = (expr);                                 \
        if (e__ != hipSuccess) return pod_hip_fail(e__, #expr);  \
    } while (0)

pod_headmap pod_make_headmap(const pod_cache *c, int layer);

// launchers (each validates nothing: the API layer did)
int pod_launch_clear_header(const pod_cache *c, hipStream_t st);
int pod_launch_reset(const pod_cache *c, int seq_slot, hipStream_t st);
int pod_launch_append(const pod_cache *c, int layer, const void *k_new, const void *v_new,
                      const int32_t *positions, int B, hipStream_t st);
int pod_launch_fill(const pod_cache *c, int layer, int seq_slot, int n, const void *k, const void *v,
                    hipStream_t st);
// sequences b_first .. b_first + B - 1; k_new, v_new: [B][T][Hkv][D] and counts: host array [B], both starting at
// sequence b_first; positions: device array indexed by sequence, or NULL (the stored lengths are the start positions)
int pod_launch_append_many(const pod_cache *c, int layer, const void *k_new, const void *v_new, const int32_t *positions,
                           const int32_t *counts, int T, int b_first, int B, hipStream_t st);
// contiguous [p0 + T][Hkv][D] keys / values / lowest layers' keys of one sequence (ks_all may be NULL)
int pod_launch_gather(const pod_cache *c, int layer, int seq_slot, int p0, int T, const void *k_chunk, const void *v_chunk,
                      const void *ks_chunk, void *k_all, void *v_all, void *ks_all, hipStream_t st);
// Chunk attention straight from the cache: stores the chunk at (layer, seq_slot) as pod_launch_append_many would, keeps the
// own keys this drops in the workspace and writes the per-tile address table pod_launch_prefill_tiles reads.  The stored
// length is left for pod_launch_prefill_tiles to change (no workgroup of the update may change what the others test).
size_t pod_chunk_direct_bytes(const pod_layout &ly, int64_t n_total, int64_t T); // workspace bytes that suffice (T <= 0: for any chunk length)
int pod_launch_chunk_update(const pod_cache *c, int layer, int seq_slot, int p0, int T, const void *k_chunk, const void *v_chunk,
                            void *workspace, size_t workspace_bytes, const unsigned long long **tile_tab, int *ntiles,
                            hipStream_t st);
int pod_launch_export(const pod_cache *c, int layer, int seq_slot, int64_t n, void *sinkK, void *sinkV,
                      void *recK, void *recV, void *distK, void *distV, hipStream_t st);
// scores == NULL: plain decode; else the score-reuse buffer (lowest layer writes, upper layers read).
// tau >= 0 (needs scores): upper layers leave the distant part out for heads whose gate reaches tau.
// step != NULL: a decode step (the new token's cache update inside the same launch); ctx is then NULL and the
// lengths in the host mirror are those before the update.
struct pod_step_args { const void *k_new, *v_new; const int32_t *positions; };
// the split-K plan of a decode launch (host logic, pod_decode.hip): waves per workgroup, tokens per distant and per
// proximal piece, distant pieces and all pieces per (sequence, kv head) pair, whether the partials are merged inside
struct pod_decode_plan_t { int waves, chunk, chunk_p, max_nd, nc; bool merge_inside; };
pod_decode_plan_t pod_plan_decode(int cus, int B, int Hkv, int P, int max_len, int env_chunk, int env_chunk_prox, bool scores,
                                  bool small_prox, bool fused_allowed, bool reader = false);
// the even split of a plain launch of several rounds (host logic, pod_decode.hip): units per workgroup, workgroups,
// units in all, partials of the (sequence, kv head) pair that is cut into most parts; unit_cum has B + 1 entries;
// unit_d = tokens per unit of distant rows (128, or 256 for an upper layer that reads logits instead of keys)
struct pod_even_plan_t { int32_t q, nwg, total, most; };
bool pod_plan_even(int slots, int B, int Hkv, int P, int unit_d, const int32_t *lens, int32_t *unit_cum, pod_even_plan_t *pl);
int pod_launch_decode(const pod_cache *c, int layer, const void *q, const void *q_shared,
                      const int32_t *ctx, int B, int max_len, float scale, void *ws, size_t ws_bytes,
                      void *scores, float tau, void *out, hipStream_t st, const pod_step_args *step = nullptr);
int pod_launch_stream_read(pod_cache *c, const void *buf, size_t bytes, hipStream_t st); // measurement aid: read bytes once, keep nothing
int pod_launch_mfma_feed(int variant, int iters, float *out, size_t out_bytes, hipStream_t st); // measurement aid (pod_probe.hip)
int pod_launch_similarity(const float *att, int L, int H, int R, int n, float *sim, hipStream_t st);
size_t pod_score_stride(const pod_layout &ly);       // fp32 elements per (sequence, query head) row
size_t pod_score_header_bytes(const pod_layout &ly); // tags, distant sums and skip flags in front of the rows
size_t pod_score_skip_offset_bytes(const pod_layout &ly); // where the skip flags int32 [B][Hq] start

// the same with keys and values located through a table: tile_tab[(stream * Hkv + kv head) * ntiles + tile] = device
// address of the first row of that head's 64-position tile, rows D * 2 bytes apart (stream 0 k, 1 v, 2 k_shared).
// Completes pod_launch_chunk_update: *len becomes n if it still is q0, else *flag is raised.
int pod_launch_prefill_tiles(const pod_layout &ly, int n, int q0, const void *q, const void *q_shared,
                             const unsigned long long *tile_tab, int ntiles, int *len, int *flag, uint64_t lowest_mask, float scale,
                             void *out, hipStream_t st);

// token selection on the distant store (pod_select.hip): scratch bytes of the three steps and their launchers.
// head_mask: kv heads to work on; votes: float [Hkv][n - S - W]; sel: int32 rows of sel_stride entries per kv head
size_t pod_select_votes_bytes(const pod_layout &ly, int64_t n, int obs);
size_t pod_select_top_bytes(const pod_layout &ly, int64_t n);
size_t pod_compact_bytes(const pod_layout &ly, int keep);
// k == NULL: the keys of positions 0 .. n - 1 are read from the cache of (layer, sequence b), which must hold n tokens
int pod_launch_select_votes(const pod_cache *c, int layer, int b, uint64_t head_mask, int n, const void *q_obs, int obs, const void *k,
                            float scale, float *votes, void *ws, hipStream_t st);
int pod_launch_select_top(int Hkv, uint64_t head_mask, const float *votes, int m, int width, int use_max, int keep,
                          float *pooled, int32_t *sel, int sel_stride, hipStream_t st);
int pod_launch_compact(const pod_cache *c, int layer, int b, int n, const int32_t *sel_all, int keep, void *ws, hipStream_t st);

size_t pod_decode_workspace_bytes(const pod_layout &ly);
// device address and size of the library's own split-K scratch array on the current device (looked up once per device)
int pod_decode_static_scratch(void **ptr, size_t *bytes);
int pod_probe_xcds(int *nxcd); // once per device: over how many XCDs one-dimensional launches spread round-robin
// lowest_mask: bit h set = kv head h takes every logit from (q, k); clear = distant logits from (q_shared, k_shared)
// k, v, k_shared: rows for positions 0 .. n-1; q, q_shared, out: rows for positions q0 .. n-1
int pod_launch_prefill(const pod_layout &ly, int layer, int n, int q0, const void *q, const void *k, const void *v,
                       const void *q_shared, const void *k_shared, uint64_t lowest_mask, float scale, void *out,
                       hipStream_t st);
