/*
 * libpod — PoD ("Proximal tokens over Distant tokens", arXiv 2412.02252) attention
 * over a split KV cache, for AMD MI355X (gfx950).  C ABI, no C++ or framework
 * types in any signature.
 *
 * The method (paper, Methodology, "Attention Sharing within Each Block"):
 * layers are grouped in blocks of consecutive layers.  For a query at position i
 * the earlier tokens are split in *proximal* tokens (the first S "sink" tokens
 * and the W most recent ones, i included) and *distant* tokens (the rest).
 * Proximal logits use the layer's own query and keys (Eq. 3, line 1); distant
 * logits are those of the block's lowest layer, i.e. that layer's query times
 * that layer's keys (Eq. 3, line 3).  One softmax runs over both sets (Eq. 4
 * and the appendix derivation show the gate form equals it) and weights the
 * layer's own values (Eq. 3, lines 2 and 4).  Consequence for storage: distant
 * keys are kept once per block, everything else per layer.
 *
 * By default blocks are uniform: layer l belongs to block l / group_size, whose
 * lowest layer is l - l % group_size; pod_config.block_lowest gives every kv head
 * its own blocks instead (the paper groups layers head by head).  GQA: query
 * head h reads KV head h / (num_q_heads / num_kv_heads).
 *
 * Conventions
 *  - Every call returns POD_OK (0) or a negative pod_status; pod_last_error()
 *    gives a thread-local message for the last failure on the calling thread.
 *  - "dev" pointers are device memory of the current HIP device, "host" pointers
 *    are ordinary host memory.  The caller owns every buffer it passes; the
 *    library never allocates or frees device memory and never synchronises the
 *    device, except pod_cache_check and pod_cache_sync_lengths (which wait on the
 *    given stream).  Every other call can be captured into a HIP graph; a captured
 *    call fixes its host-side arguments, the mirror's lengths (below) among them,
 *    so a graph is replayed from the cache state it was captured at.
 *  - A cache handle keeps host-side state (the mirror): use it from one host thread
 *    at a time.
 *  - All device work is enqueued on the stream argument (a hipStream_t passed as
 *    void*; NULL = the default stream).  Calls that touch one cache must be
 *    issued in program order on one stream (or be ordered by the caller).
 *  - Tensors are bf16 (raw 16-bit, round-to-nearest-even where the library
 *    rounds), contiguous, row-major with the last index fastest.
 *  - head_dim must be 64 or 128; num_q_heads / num_kv_heads must be <= 16.
 *  - Sequences live in slots 0 .. max_batch-1.  A batched call with B entries
 *    addresses slots 0 .. B-1 (entry b <-> slot b).
 *  - The library mirrors each (layer, slot) length on the host from the calls it
 *    has seen, to validate arguments.  Contracts it cannot see from the host
 *    (values inside device arrays) are checked inside the kernels: a violating
 *    entry is skipped (nothing written for it, output rows zeroed), a sticky flag
 *    is raised in device memory, and pod_cache_check reports it.  No input can
 *    make a kernel read or write outside the buffers described here.
 */
#ifndef POD_H
#define POD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum pod_status {
    POD_OK = 0,
    POD_ERR_INVALID_ARG = -1, /* bad pointer, index, shape or unsupported configuration */
    POD_ERR_CAPACITY = -2,    /* more tokens / sequences / bytes than the buffer was sized for */
    POD_ERR_STATE = -3,       /* call does not fit the cache's state (e.g. fill of a non-empty slot) */
    POD_ERR_HIP = -4          /* the HIP runtime reported an error */
} pod_status;

typedef struct pod_config {
    int32_t num_layers;   /* L, a multiple of group_size */
    int32_t group_size;   /* G: layers per block; G = 1 is ordinary attention */
    int32_t num_q_heads;  /* Hq */
    int32_t num_kv_heads; /* Hkv, divides Hq, at most 64 */
    int32_t head_dim;     /* d: 64 or 128 */
    int32_t sink;         /* S = n_s >= 0 */
    int32_t window;       /* W = n_r >= 1; counts the query's own token */
    int32_t max_batch;    /* sequence slots */
    int32_t max_context;  /* tokens per sequence the buffers are sized for */
    /*
     * Optional head-wise blocks (the paper groups layers head by head, "Greedy Layer Grouping
     * Algorithm"; per kv head under GQA): host array int32 [num_layers][num_kv_heads], entry
     * (l, h) = lowest layer of the block layer l belongs to for kv head h.  Blocks are runs of
     * consecutive layers: entry (0, h) = 0 and entry (l, h) is entry (l-1, h) or l.  NULL: uniform
     * blocks of group_size layers.  Read during the call only (the cache keeps a copy).  With a table, group_size is ignored, and for a layer that is not the lowest
     * of every head's block the callers of decode / prefill pass q_shared (and k_shared)
     * gathered head by head: the slice of head h comes from layer entry (l, h).
     */
    const int32_t *block_lowest;
} pod_config;

typedef struct pod_cache pod_cache; /* host-side handle; holds no device allocation of its own */

/* Message for the last error on this thread ("" if none).  Never NULL. */
const char *pod_last_error(void);

/*
 * Bytes of device memory a cache for cfg needs (all regions at max_context, plus
 * a small header of per-sequence lengths and the error flag).  host out.
 */
int pod_cache_bytes(const pod_config *cfg, size_t *bytes);

/*
 * The paper's memory accounting for one sequence holding n tokens: bytes of K/V
 * actually live in the PoD cache (distant keys once per block: abstract, Eq. 3)
 * and in a dense cache (K and V of every token at every layer).  host outs.
 *   pod   = 2*d*Hkv * [ L*(2*min(n,S+W) + n_dist) + (L/G)*n_dist ],  n_dist = max(0, n-S-W)
 *   dense = 2*d*Hkv * 2*L*n
 */
int pod_cache_live_bytes(const pod_config *cfg, int64_t n, size_t *pod_bytes, size_t *dense_bytes);

/*
 * Lay a cache out in dev_buf (device memory, 256-byte aligned, >= pod_cache_bytes).
 * Enqueues a clear of the header on stream; K/V regions are left as they are
 * (never read before written).  *out receives the handle.
 */
int pod_cache_init(const pod_config *cfg, void *dev_buf, size_t bytes, void *stream, pod_cache **out);

/* Free the host handle.  The device buffer stays the caller's. */
int pod_cache_destroy(pod_cache *cache);

/* Forget the contents of slot seq_slot (or of every slot if seq_slot < 0) at every layer. */
int pod_cache_reset(pod_cache *cache, int seq_slot, void *stream);

/* Host mirror of the number of tokens stored for (layer, seq_slot).  host out. */
int pod_cache_seq_len(const pod_cache *cache, int layer, int seq_slot, int64_t *n);

/*
 * Sizes of the three regions (layer, seq_slot) holds by the host mirror's length n, in tokens:
 * counts[0] sink tokens (positions below S), counts[1] tokens in the recent window (the last
 * min(W, n - S) positions), counts[2] distant tokens (everything between); *has_distant_keys
 * (may be NULL) = 1 if `layer` is the lowest layer of some kv head's block, i.e. keeps distant keys.
 * These are the row counts pod_cache_export_logical writes.  host outs.
 */
int pod_cache_region_counts(const pod_cache *cache, int layer, int seq_slot, int64_t counts[3], int *has_distant_keys);

/*
 * Wait for stream, then report whether any kernel since the last check skipped an
 * entry because a device-side contract was violated (wrong position, wrong
 * context length, overflow): POD_ERR_STATE if so (the flag is cleared), else POD_OK.
 * The host mirror counts every entry of every accepted call, skipped ones included, so after a
 * POD_ERR_STATE from here it may be ahead of the device: call pod_cache_sync_lengths before going on.
 */
int pod_cache_check(pod_cache *cache, void *stream);

/*
 * Wait for stream, then copy the device-side lengths of every (layer, slot) into the host
 * mirror.  Only needed after work the host did not see call by call: a replay of a captured
 * HIP graph advances the device-side lengths but not the mirror (a captured call fixes its
 * host-side arguments, the mirror's lengths among them, so a graph must be replayed from the
 * cache state it was captured at).
 */
int pod_cache_sync_lengths(pod_cache *cache, void *stream);

/* Bytes of device scratch pod_decode_attention needs for cfg (split-K partial results). host out. */
int pod_workspace_bytes(const pod_config *cfg, size_t *bytes);

/*
 * Cache update at decode time (derived from Eq. 3's index ranges): one new token per
 * sequence enters `layer`.
 *   k_new, v_new : dev bf16 [B][Hkv][d]
 *   positions    : dev int32 [B]; positions[b] must equal the number of tokens slot b
 *                  already holds at this layer (checked in the kernel)
 * Token p goes to sink slot p if p < S, else into the ring of W recent tokens.
 * If the ring is full, the token it displaces (position p-W) becomes distant first:
 * its value moves to this layer's distant-V store, and its key moves to the block's
 * distant-K store only if `layer` is the block's lowest layer (other layers drop it).
 * POD_ERR_CAPACITY if the host mirror shows a slot already at max_context.
 */
int pod_cache_append(pod_cache *cache, int layer, const void *k_new, const void *v_new,
                     const int32_t *positions, int B, void *stream);

/*
 * Cache construction from a whole prompt; same result as n appends.
 *   k, v : dev bf16 [n][Hkv][d], positions 0..n-1 of slot seq_slot at `layer`
 * The slot must be empty at this layer (POD_ERR_STATE otherwise); n <= max_context.
 */
int pod_cache_fill(pod_cache *cache, int layer, int seq_slot, int n, const void *k, const void *v,
                   void *stream);

/*
 * Decode attention (Eq. 3 + Eq. 4 as one joint softmax), one query token per sequence,
 * over what the cache holds for `layer` after the token's own K/V was appended.
 *   q            : dev bf16 [B][Hq][d], this layer's query
 *   q_shared     : dev bf16 [B][Hq][d], the query of the block's lowest layer for the
 *                  same token; may be NULL when `layer` is the lowest layer of its block
 *                  (then q serves).  Passing q itself on an upper layer gives the
 *                  "shared keys, own queries" variant, which is not the paper's rule.
 *   context_lens : dev int32 [B]; tokens held for slot b including the query's own;
 *                  0 skips the entry (output row zeroed); any other value must equal the
 *                  cache's length for (layer, slot b) (checked in the kernel)
 *   max_context_len : host upper bound on context_lens (sizes the launch); 0 = use the
 *                  host mirror's maximum over the B slots.  An entry with a larger
 *                  context_lens is skipped like any other contract violation (output row
 *                  zeroed, flag raised)
 *   scale        : logits multiplier, 1/sqrt(d) in the paper
 *   workspace    : dev scratch of >= pod_workspace_bytes(cfg); contents undefined afterwards
 *   out          : dev bf16 [B][Hq][d]
 * The block's lowest layer must hold the same number of distant tokens as `layer`
 * (append/fill the lowest layer first).
 */
int pod_decode_attention(pod_cache *cache, int layer, const void *q, const void *q_shared,
                         const int32_t *context_lens, int B, int max_context_len, float scale,
                         void *workspace, size_t workspace_bytes, void *out, void *stream);

/*
 * One decode step of a layer in one launch: pod_cache_append(layer, k_new, v_new, positions) followed by
 * pod_decode_attention(layer, q, q_shared, context_lens = positions + 1): same cache contents afterwards
 * (bit for bit) and the same attention (Eq. 3 + Eq. 4 over the tokens including the new one).  The kernel
 * walks the rows held before the call; one workgroup per (sequence, kv head) also takes the new token
 * (proximal: this layer's query and the new key) and the token it displaces from the recent window
 * (distant from now on: the key the block's lowest layer holds for it, with that layer's query) and
 * performs the cache update.  Where the launch is about one resident round of workgroups the last
 * workgroup to finish merges the partial results; larger launches are followed by the merging kernel.
 *   k_new, v_new : dev bf16 [B][Hkv][d];  positions : dev int32 [B], as in pod_cache_append
 *   q, q_shared, scale, workspace, out : as in pod_decode_attention
 *   max_context_len : host upper bound on positions + 1; 0 = the host mirror's maximum + 1
 * Every entry takes a token (no inactive entries).  A wrong position skips the entry: nothing
 * stored, output row zeroed, flag raised (pod_cache_check).  The block's lowest layer must take the
 * token before the block's upper layers.
 */
int pod_decode_step(pod_cache *cache, int layer, const void *k_new, const void *v_new, const void *q,
                    const void *q_shared, const int32_t *positions, int B, int max_context_len, float scale,
                    void *workspace, size_t workspace_bytes, void *out, void *stream);

/*
 * pod_decode_step with score reuse (the reading of Eq. 3 line 3 in which a block's upper layers take the lowest layer's
 * distant attention scores instead of recomputing them from the shared keys): pod_cache_append(layer, ...) followed by
 * pod_decode_attention_reuse(layer, q, context_lens = positions + 1, ..., scores), same cache contents and the same
 * attention.  Call it for the block's lowest layer first (it writes the scaled distant logits of this token's query
 * into `scores`, among them the logit of the token the new one displaces from the window), then for the block's
 * upper layers with the same `scores` (they stream values, proximal keys and those logits only).
 * One streaming launch per layer (two for a layer whose kv heads are of both kinds under a head-wise block table),
 * followed by the merging kernel where the launch is several rounds of workgroups.  Arguments as in pod_decode_step
 * and pod_decode_attention_reuse.
 * Errors and device-side checks as there; logits left by this call carry no distant sums, so a later
 * pod_decode_attention_gated on an upper layer refuses them (flag) - use pod_decode_attention_gated at the lowest layer
 * for that.
 */
int pod_decode_step_reuse(pod_cache *cache, int layer, const void *k_new, const void *v_new, const void *q,
                          const int32_t *positions, int B, int max_context_len, float scale, void *workspace,
                          size_t workspace_bytes, void *scores, size_t scores_bytes, void *out, void *stream);

/*
 * Where the decode kernels take sequence lengths from.  0 (default): batches of up to 256
 * sequences pass the host mirror's lengths as kernel arguments (the shortest way to the first
 * load; the device-side arrays are still compared with them).  1: only from the device arrays the
 * calls name (context_lens, positions) and the cache's own header; nothing a call enqueues then
 * depends on the mirror, so a HIP graph captured over pod_cache_append / pod_decode_attention /
 * pod_decode_step / pod_decode_step_reuse calls can be replayed for successive tokens: refresh the device arrays between
 * replays, pass max_context_len >= every length the replays will see (it sizes the launch and must
 * be given), always pass q_shared for an upper layer, and call pod_cache_sync_lengths once the
 * replays are done.  Checks the host can no longer make are made on the device (flag).
 */
int pod_cache_set_length_source(pod_cache *cache, int from_device);

/*
 * How this cache's decode launches are shaped on the current device (host out, for reports and tests):
 * info[0] = number of XCDs a one-dimensional launch was seen to spread over round-robin (0 = no such
 * pattern); info[1] = 1 if split-K partials are handed over inside one XCD's L2 where the batch allows;
 * info[2] = 1 if plain decode merges its partials inside the streaming kernel; info[3] = the length source
 * (pod_cache_set_length_source).
 */
int pod_cache_launch_info(const pod_cache *cache, int32_t info[4]);

/*
 * pod_decode_attention for callers that cannot allocate device memory or take a workspace from
 * an allocator: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, kernels and results as pod_decode_attention, except that the
 * split-K partial results go to a fixed 16 MiB array inside the library's code object (one copy per
 * GPU, held until the process ends; its device address is looked up in pod_cache_init) instead of
 * a caller's workspace.  The call allocates and frees nothing.
 *  - POD_ERR_CAPACITY if this call's launch needs more than the 16 MiB: it needs
 *    4 * B * num_q_heads * chunks * (head_dim + 2) bytes, chunks = the split-K pieces of the longest
 *    sequence (pod_decode_plan gives their number).  With 32 query heads x 128: batch 1 at 32K tokens takes
 *    0.6 MB, 16 sequences of up to 32K tokens 8.8 MB, 4 sequences of 128K tokens 8.6 MB.  Larger
 *    launches go through pod_decode_attention.
 *  - Every call on one GPU shares that GPU's array: calls that overlap in time on one GPU (other
 *    streams, other caches, other host threads) race; issue them in order on one stream.
 *  - The current device must be the cache's.
 */
int pod_decode_attention_static(pod_cache *cache, int layer, const void *q, const void *q_shared,
                                const int32_t *context_lens, int B, int max_context_len, float scale,
                                void *out, void *stream);

/*
 * Decode attention with score reuse: same result as pod_decode_attention, but the distant
 * logits are computed once per block.  Eq. 3 line 3 defines the distant logits of every layer of
 * a block as those of the block's lowest layer; called for the lowest layer, this entry point
 * also writes them (scaled, fp32) to `scores`; called for an upper layer it reads them from
 * there instead of streaming the block's distant keys again, which cuts the bytes such a call
 * has to read from 2*n rows to about n rows + 4 bytes per (query head, distant token).
 *   scores : dev buffer of >= pod_score_buffer_bytes(cfg), 256-byte aligned, holding for every
 *            kv head the logits of ONE block at a time: call the layers in ascending order for
 *            the same token, batch and scale (a block's lowest layer first, then its upper
 *            layers, before the next block).  A tag in the buffer (token count, block and
 *            scale, per sequence and kv head) is checked on the device; a mismatch zeroes the
 *            output row and raises the flag pod_cache_check reports.
 * With head-wise blocks (pod_config.block_lowest) a layer can be the lowest for some kv heads
 * and an upper layer for others: each kv head writes or reads its own part of the buffer.
 * Other arguments as in pod_decode_attention; no q_shared is needed.
 */
int pod_score_buffer_bytes(const pod_config *cfg, size_t *bytes);
int pod_decode_attention_reuse(pod_cache *cache, int layer, const void *q, const int32_t *context_lens, int B,
                               int max_context_len, float scale, void *workspace, size_t workspace_bytes,
                               void *scores, size_t scores_bytes, void *out, void *stream);

/*
 * Decode attention with the gated skip of distant tokens (appendix "Computation Optimization for
 * Distant Tokens").  Built on score reuse: same `scores` buffer and call order.  For the block's
 * lowest layer the call equals pod_decode_attention_reuse (it also leaves the distant
 * maximum and sum of every query head in the buffer).  For an upper layer (head by head with
 * head-wise blocks) the gate of Eq. 4,
 *     g = sum exp(a^P) / (sum exp(a^P) + sum exp(a^D)),
 * is evaluated per (sequence, query head) once the proximal logits are known; heads with
 * g >= tau leave the distant tokens out and return o^P, the softmax over their proximal tokens
 * alone; the distant rows of a kv head are not read at all when all of its query heads skip.
 *   tau : in [0, 1].  1 never skips (g < 1 whenever distant tokens exist); 0 always skips.
 * The decision is taken in fp32 from bf16-input logits: a head whose g lies within rounding of
 * tau may fall on either side.  pod_score_skip_offset gives the byte offset inside `scores` of
 * the int32 [max_batch][num_q_heads] flags (1 = distant part left out) written by the last upper-layer call.
 */
int pod_decode_attention_gated(pod_cache *cache, int layer, const void *q, const int32_t *context_lens, int B,
                               int max_context_len, float scale, float tau, void *workspace,
                               size_t workspace_bytes, void *scores, size_t scores_bytes, void *out, void *stream);
int pod_score_skip_offset(const pod_config *cfg, size_t *offset);

/*
 * Inter-layer attention similarity for the offline grouping ("Attention Similarity Measurement"):
 * sim[h][a][b] = 1 - mean over the sampled rows of the Jensen-Shannon divergence (base-2
 * logarithms, so in [0, 1]) between the attention rows of layers a and b for head h; 1 on the
 * diagonal.  One GPU pass over the rows per layer pair.
 *   att : dev float [num_layers][num_heads][rows][n], every row a probability vector (the last
 *         `q` tokens of `N` samples flattened into rows = N * q); 16-byte aligned, rows * n a
 *         multiple of 4
 *   sim : dev float [num_heads][num_layers][num_layers], fully written
 * Feed sim (copied to the host) to pod_group_layers.
 */
int pod_layer_similarity(const float *att, int num_layers, int num_heads, int rows, int n, float *sim, void *stream);

/*
 * Offline grouping of layers into head-wise blocks ("Greedy Layer Grouping Algorithm"; host
 * arrays, no GPU work).  sim: float [num_q_heads][num_layers][num_layers], sim[h][a][b] the
 * attention similarity of layers a and b for query head h.  For each kv head, bottom-up: layer
 * l joins the current block if it is similar to ALL layers already in it, else it starts a new
 * block; two layers are similar for a kv head if sim >= threshold for more than half of its
 * query heads (the paper's majority vote under GQA; a tie is not a majority; with one query
 * head per kv head this is the plain test).  lowest_out: int32 [num_layers][num_kv_heads], in
 * the form pod_config.block_lowest takes.
 */
int pod_group_layers(const float *sim, int num_layers, int num_q_heads, int num_kv_heads, float threshold,
                     int32_t *lowest_out);

/*
 * Prefill attention for one sequence (Eq. 3 with the window taken at each query's own
 * position: key j is proximal for query i if j < S or j > i - W), causal, joint softmax.
 *   q        : dev bf16 [n][Hq][d];  k, v : dev bf16 [n][Hkv][d] of `layer`
 *   q_shared, k_shared : the lowest layer's q and k (same shapes); both NULL when `layer`
 *              is the lowest of its block
 *   out      : dev bf16 [n][Hq][d]
 *   write_cache : nonzero = also build the cache for (layer, seq_slot) from k, v as
 *              pod_cache_fill does (slot must be empty at this layer); with 0 the cache
 *              is not touched and seq_slot is ignored
 */
int pod_prefill_attention(pod_cache *cache, int layer, int seq_slot, int n, const void *q, const void *k,
                          const void *v, const void *q_shared, const void *k_shared, float scale,
                          void *out, int write_cache, void *stream);

/*
 * Cache update with several tokens per sequence in one call (a chunk of a prompt, or tokens
 * accepted together; the state the index ranges of Eq. 3 give after all of them, i.e. the
 * state after appending them one at a time).
 *   k_new, v_new : dev bf16 [B][T][Hkv][d]
 *   positions    : dev int32 [B], position of each sequence's first new token; must equal the
 *                  number of tokens the slot holds at this layer (checked in the kernel;
 *                  ignored for sequences that take no token)
 *   counts       : HOST int32 [B] or NULL: sequence b takes its first counts[b] rows
 *                  (0 <= counts[b] <= T; NULL = T for all)
 * New tokens that are outside the window of W recent tokens by the end of the call go to the
 * distant stores directly (key only where `layer` is the lowest of the head's block); the
 * others enter the ring, whose displaced tokens become distant as in pod_cache_append.
 * POD_ERR_CAPACITY if the host mirror shows a slot would exceed max_context.
 */
int pod_cache_append_many(pod_cache *cache, int layer, const void *k_new, const void *v_new,
                          const int32_t *positions, const int32_t *counts, int T, int B, void *stream);

/* Bytes of device scratch that suffice for pod_prefill_attention_chunk on a sequence that holds
 * n_total tokens after the chunk, whichever way the call takes (see there). host out. */
int pod_prefill_chunk_workspace_bytes(const pod_config *cfg, int64_t n_total, size_t *bytes);
/* The smaller scratch that suffices when the call takes its first way (see there) for a chunk of
 * T tokens that brings the sequence to n_total: for callers that always store the chunk, lowest
 * layers first.  A call that needs more than it is given returns POD_ERR_CAPACITY. host out. */
int pod_prefill_chunk_in_place_bytes(const pod_config *cfg, int64_t n_total, int64_t T, size_t *bytes);

/*
 * Prefill attention for a chunk of T new tokens of a sequence whose first p0 tokens are in
 * the cache already (a prompt processed in pieces; p0 = tokens (layer, seq_slot) holds, p0 = 0
 * is pod_prefill_attention).  Chunk token t has position p0 + t and attends positions
 * j <= p0 + t by Eq. 3 taken at its own position: proximal keys (j < S or j > p0 + t - W) from
 * this layer, distant keys from the lowest layer of the head's block with that layer's query;
 * values from this layer; one joint softmax.
 *   q        : dev bf16 [T][Hq][d];  k, v : dev bf16 [T][Hkv][d] of `layer` for the chunk
 *   q_shared, k_shared : the lowest layer's q and k for the chunk (same shapes); both NULL when
 *              `layer` is the lowest of its block for every kv head
 *   workspace: dev scratch of pod_prefill_chunk_workspace_bytes(cfg, p0 + T) bytes, 256-byte aligned
 *   out      : dev bf16 [T][Hq][d]
 *   write_cache : nonzero = store the chunk at (layer, seq_slot) as pod_cache_append_many does
 * Keys of earlier positions come from the cache: this layer's sink and recent window, and the
 * stores of the lowest layer of each head's block, which must hold either p0 tokens or
 * p0 + T (it has stored this chunk already): otherwise POD_ERR_STATE.
 *
 * Two ways, same result.  With write_cache set and the lowest layers already at p0 + T (the
 * usual order: every layer takes the chunk, lowest layers first) the chunk is stored FIRST and
 * the attention kernel reads keys and values where the cache holds them; the workspace then
 * carries only the own keys that this update drops but the chunk's queries still see inside
 * their windows (at most T rows per kv head), a few staged 64-row tiles and a table of tile
 * addresses.  If the stored length on the device is not p0 (a host mirror that ran ahead),
 * nothing is stored, `out` is undefined and the sticky flag is raised, as in
 * pod_cache_append_many.  Otherwise (write_cache 0, a lowest layer still at p0, or
 * POD_CHUNK_IN_PLACE=0 in the environment when the cache was created) keys and values of all
 * p0 + T positions are first copied into the workspace as contiguous arrays and the chunk is
 * stored afterwards if asked.  k_shared is not read on the first way: the lowest layer's cache
 * holds the same rows.
 */
int pod_prefill_attention_chunk(pod_cache *cache, int layer, int seq_slot, int T, const void *q, const void *k,
                                const void *v, const void *q_shared, const void *k_shared, float scale,
                                void *workspace, size_t workspace_bytes, void *out, int write_cache, void *stream);

/*
 * Token selection on the distant store: the combination with a token-selection method that the
 * result tables list as "PoD+SnapKV" (appendix section on SnapKV: observation window of 64 prompt
 * positions, grouped-query attention).  The paper gives no rule of its own; these calls apply the
 * published one to the tokens the combination can drop, the distant ones (proximal tokens are
 * kept in full by definition, Section 3), per block of layers and kv head, since a block shares
 * the keys and the logits of its distant tokens (Eq. 3):
 *   1. pod_select_votes at a block's lowest layer, once the prompt's q and k of that layer exist:
 *      votes[h][t] = attention that distant token S + t receives from the queries of the last
 *      `obs` prompt positions in the query heads of kv head h's group, each in its joint softmax
 *      over the keys up to its own position (Eq. 4), summed.  fp32, fixed summation order.
 *   2. pod_select_top: votes pooled over pool_width neighbours (POD_POOL_AVG: window sum /
 *      pool_width with zeros outside the distant range; POD_POOL_MAX: maximum over the positions
 *      that exist), then the `keep` largest per kv head (of equal ones the earlier token), written
 *      as ascending distant indices t to row (layer, h) of sel.
 *   3. pod_cache_compact for every layer, after the prompt is stored at it: the selected
 *      distant rows move to the front of the layer's distant stores (keys only where it keeps
 *      them), the recent ring is turned, and the stored length of (layer, seq_slot) becomes
 *      S + keep + W.  From then on the cache is that of the shorter sequence: positions passed to
 *      the append, step and decode calls count stored tokens, S + keep + W, S + keep + W + 1, ...
 *      (rotary positions are the caller's and unaffected: keys arrive rotated).
 * Shapes (all device memory unless said otherwise):
 *   q_obs : bf16 [obs][Hq][d], queries of prompt positions n - obs .. n - 1 at `layer`;  1 <= obs <= W
 *   k     : bf16 [n][Hkv][d], the prompt's keys at `layer` (what pod_prefill_attention was given), or
 *           NULL: the keys are read where the cache holds them; (layer, seq_slot) must then hold the
 *           n prompt tokens (POD_ERR_STATE otherwise) -- the way for a prompt that was stored in chunks.
 *           The votes are the same bits either way.  seq_slot is not used when k is given.
 *   votes : float [Hkv][n - S - W]; rows of kv heads whose block does not start at `layer` are
 *           neither written (votes) nor read (top).  pod_select_top takes any finite floats (what
 *           pod_select_votes writes is >= 0); its result for rows that hold NaNs is unspecified
 *   sel   : int32 [num_layers][Hkv][keep]; pod_select_top writes rows (layer, h) of the heads whose
 *           block starts at `layer`; pod_cache_compact reads, for head h, the row of the lowest
 *           layer of h's block.  1 <= keep <= n - S - W.
 *   workspace : 256-byte aligned scratch of pod_select_workspace_bytes(cfg, n, obs, keep) bytes
 *           (host out; the maximum over the three calls), contents undefined afterwards
 * n is the prompt length (votes, top) and must equal the stored length at compaction, which is
 * taken from the host mirror; a device-side length that differs, or a sel entry outside
 * [0, n - S - W), raises the sticky flag (pod_cache_check): a length that differs leaves the cache
 * untouched, a bad entry is replaced by 0.  POD_ERR_INVALID_ARG for shapes outside the limits above or
 * a layer that starts no block (votes, top), POD_ERR_STATE for a slot without distant tokens,
 * POD_ERR_CAPACITY for a workspace that is too small.
 */
#define POD_POOL_AVG 0
#define POD_POOL_MAX 1
int pod_select_workspace_bytes(const pod_config *cfg, int64_t n, int obs, int keep, size_t *bytes);
int pod_select_votes(pod_cache *cache, int layer, int seq_slot, int n, const void *q_obs, int obs, const void *k,
                     float scale, float *votes, void *workspace, size_t workspace_bytes, void *stream);
int pod_select_top(pod_cache *cache, int layer, int n, const float *votes, int pool_width, int pool_kind, int keep,
                   int32_t *sel, void *workspace, size_t workspace_bytes, void *stream);
int pod_cache_compact(pod_cache *cache, int layer, int seq_slot, const int32_t *sel, int keep, void *workspace,
                      size_t workspace_bytes, void *stream);

/*
 * Test hook: copy the cache's logical content for (layer, seq_slot) out in position
 * order, each as dev bf16 [tokens][Hkv][d]:
 *   sink   : positions [0, min(n,S))           recent : [max(S, n-W), n), oldest first
 *   dist   : positions [S, n-W)                (distK only at a block's lowest layer)
 * Any pointer may be NULL (skipped).  Asking distK of an upper layer is POD_ERR_INVALID_ARG.
 * n is the host mirror's length; buffers must hold that many rows per region.
 */
int pod_cache_export_logical(pod_cache *cache, int layer, int seq_slot, void *sinkK, void *sinkV,
                             void *recentK, void *recentV, void *distK, void *distV, void *stream);

/*
 * Measurement aid: while enabled, pod_decode_attention brackets its dominant kernel (the
 * split-K partial kernel that streams K and V) with HIP events on the call's stream, up to
 * max_records launches.  pod_profile_read waits for the recorded events and returns the
 * summed kernel time in milliseconds and the number of launches, then forgets them.
 * Events are host objects: no device memory is allocated.  Do not enable while the stream is
 * being captured into a graph.
 */
int pod_profile_enable(pod_cache *cache, int max_records);
int pod_profile_disable(pod_cache *cache);
int pod_profile_read(pod_cache *cache, double *total_ms, int *launches);
/* The same, launch by launch: ms_each (host float [capacity]) receives the kernel time of each recorded launch in
 * call order, *launches how many were written; the records are then forgotten. */
int pod_profile_read_each(pod_cache *cache, float *ms_each, int capacity, int *launches);
/*
 * Measurement aid for the prefill kernel's roofline: a synthetic loop of 32x32x16 bf16 MFMAs on every CU at the
 * prefill kernel's occupancy (two waves per SIMD), timed by the caller.  variant 0: MFMAs only; 1: each MFMA takes one
 * operand fragment (1 KB per wave) out of LDS; 2: the same plus 3 fma + 1 exponential per MFMA (about the kernel's
 * vector work); 3: one LDS fragment per two MFMAs, same vector work.  Each SIMD executes
 * iters * 16 (variant 3: * 32) MFMAs; 13.6 ns per MFMA and SIMD = the pipe never idles.  dev_out: scratch of at least
 * 2048 * (number of CUs) bytes, contents undefined afterwards.
 */
int pod_profile_mfma_feed(int variant, int iters, void *dev_out, size_t out_bytes, void *stream);

/*
 * Host logic, no device needed: how a plain pod_decode_attention / pod_decode_step launch for `batch` sequences of up
 * to max_context_len tokens is cut into split-K pieces on a device with num_cus compute units, without tuning
 * overrides (proximal_rows = sink + window).  plan[0] waves per workgroup, plan[1] tokens per distant piece, plan[2]
 * tokens per proximal piece, plan[3] distant pieces per (sequence, kv head) pair, plan[4] all pieces per pair,
 * plan[5] 1 if the last workgroup of a pair merges the partials inside the launch, 0 if a second kernel does.
 * Pieces are whole tiles of 32 tokens and cover the regions; plan[4] never exceeds what pod_workspace_bytes provides for.
 * Returns POD_ERR_INVALID_ARG for non-positive arguments or a NULL plan.
 */
int pod_decode_plan(int num_cus, int batch, int num_kv_heads, int proximal_rows, int max_context_len, int32_t plan[6]);

/*
 * Host logic, no device needed: the even split a launch takes where pod_decode_plan's plan[5] is 0 and the host
 * knows the lengths (batch <= 256, lengths not taken from the device): plain launches, and score-reuse decode steps
 * of layers none of whose kv heads starts a block (they read logits).  context_lens: HOST int32 [batch], tokens each sequence holds (<= 0:
 * none).  The rows of the batch stand in one line - sequence after sequence, inside a sequence kv head after kv head,
 * inside such a pair its distant rows (tokens beyond proximal_rows), then its proximal rows - counted in units:
 * distant_unit_tokens distant rows (128; 256 for a score-reuse step of an upper layer, whose distant rows cost about
 * half the bytes), 128 proximal rows; a region's last unit may be short.  unit_cum: HOST out int32 [batch + 1],
 * units per kv head of the sequences before b.  plan[0] units per workgroup q (workgroup w walks units
 * [w q, (w + 1) q) of the line), plan[1] workgroups, plan[2] units in all, plan[3] the largest number of workgroups
 * that share one (sequence, kv head) pair = partial results per pair; all 0 if no sequence holds a token.
 */
int pod_decode_even_plan(int num_cus, int batch, int num_kv_heads, int proximal_rows, int distant_unit_tokens,
                         const int32_t *context_lens, int32_t plan[4], int32_t *unit_cum);

/*
 * Measurement aid: while dev_buf is set (NULL = off), every workgroup of a pod_decode_step / fused
 * pod_decode_attention launch that stores a partial result leaves 8 uint64 words in it, at index (workgroup number
 * in the launch) * 8: (sequence * num_kv_heads + kv head) << 32 | piece (bit 31 set: this workgroup merged), the id of
 * the XCD it ran on, and the device's 100 MHz clock at its start, at the end of its tile loop, when its partial was
 * stored, when its arrival was counted, and at its end.  Launches whose partials a second kernel merges record too:
 * words 0, 2, 3 and 6 as above (start, end of the tile loop, end), word 1 = XCD id | hardware id register << 8 (which
 * CU); an even-split launch (pod_decode_even_plan) records per walking workgroup its number, that word 1, and the
 * clock at its start (words 2 and 3) and end (word 6).  bytes / 64 workgroups are recorded; later launches overwrite
 * earlier ones.  The caller owns dev_buf.
 */
int pod_profile_set_trace(pod_cache *cache, void *dev_buf, size_t bytes);

/*
 * Measurement aid: enqueue the plainest possible kernel that reads `bytes` of device memory once (16-byte
 * non-temporal loads, one resident round of workgroups, nothing stored).  Timed by the caller on memory that is not in any cache, it
 * gives the rate a streaming launch of that size can reach on this device: the ceiling the decode kernel's
 * launches are compared with.  dev_buf 16-byte aligned, bytes a positive multiple of 16.  With a cache whose
 * profiling is enabled (cache may be NULL) the launch is recorded like a decode launch: same events, read back
 * through pod_profile_read / pod_profile_read_each.
 */
int pod_profile_stream_read(pod_cache *cache, const void *dev_buf, size_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* POD_H */
