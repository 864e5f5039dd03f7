// Decode attention over the split cache: split-K flash decoding on gfx950.
//
// One query token per sequence (Eq. 3 of the paper with i = n-1) and one joint softmax over
// proximal and distant tokens (Eq. 4 / appendix derivation).  The token axis of every
// (sequence, kv head) pair is cut in chunks; a workgroup reduces one chunk to a partial
// (running max m, normaliser l, unnormalised output acc) and the partials are merged by the
// last workgroup of the pair to finish (launches of about one resident round of workgroups) or
// by a second kernel (larger launches).  The merge of two partials is exactly the paper's gate:
// with l_P, l_D the two normalisers brought to a common max, g = l_P / (l_P + l_D).
// A decode step (pod_decode_step) also performs the new token's cache update inside the launch.
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
#include <stddef.h>

#include <mutex>

#include "pod_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4; // native 128-bit vector (plain loads/stores, no struct copies)

constexpr int kWaves = 4;          // waves per workgroup ...
// ... but 8 where the last workgroup of a (sequence, kv head) pair merges the partials: that merge is one CU reading
// every partial of the pair, which goes the faster the fewer and larger the pieces are and the more waves read
// (measured, one workgroup reading 128 KB it finds in the L2: 4 waves 1.7 us, 8 waves 0.9 us).
constexpr int fuse_waves(int fuse) { return fuse == 1 || fuse == 2 ? 8 : kWaves; }
constexpr int kTile = 32;          // tokens per wave iteration
constexpr float kNegBig = -1.0e30f; // stands in for -inf (keeps exp2 arguments finite)
constexpr int kMinChunk = 128;     // smallest chunk (tokens) a workgroup takes
constexpr int kMaxHostLens = 256;  // batch sizes up to this pass the host mirror's lengths as kernel arguments
constexpr int kUnit = kWaves * kTile; // tokens of one step of a four-wave workgroup: the unit the even split counts in
// ... for distant rows of an upper layer with score reuse twice as many: such a row costs a value row and its logits, 17/32
// of the bytes of a row whose key is read as well, so that all units cost about the same
__host__ __device__ constexpr int even_unit_distant(int mode) { return mode == 2 ? 2 * kUnit : kUnit; }

// Kernel arguments.  Everything is resolved on the host so that the kernel's way to its first
// K/V load is short: the fields a workgroup needs for its first load addresses sit at the start
// of the argument block, and with the host mirror's sequence length among the arguments no
// device memory has to be read first (a dependent load there costs 1-8 us once the other
// workgroups saturate the memory system).
struct decode_hot { // exactly two 64-byte lines, read in one go at kernel entry
    // line 0: what a workgroup needs for its first load addresses
    const u32x4 *kdist, *vdist, *kprox, *vprox; // row 0 of (slot 0, head 0) in this layer's / block's regions
    int32_t cd, prows;   // rows per (slot, head) in the distant / proximal regions (Cd, P = S + W)
    int32_t hkv, rep;
    int32_t chunk;       // tokens per workgroup: distant chunks in the low 16 bits, proximal chunks in the high 16 bits
    int32_t max_nd;      // distant chunk slots per (sequence, head)
    int32_t nc;          // all chunk slots per (sequence, head): max_nd + proximal slots
    int32_t use_hlen;    // 1: hlen[] holds the host mirror's length of every slot < B
    // line 1: queries, partial results, device-side lengths
    const pod_bf16 *q, *q_shared;
    float scale_log2e;
    int32_t hq;
    float *part_acc; // [B][Hq][nc][D]
    float *part_ml;  // [B][Hq][nc][2]
    const int32_t *ctx;         // context_lens
    const int32_t *lens_layer;  // device-side lengths of this layer   [B]
    const int32_t *lens_lowest; // ... of the block's lowest layer     [B]
};
static_assert(sizeof(decode_hot) == 128, "decode_hot must be two 64-byte lines");

struct decode_params {
    decode_hot hot;
    int32_t *flag;
    int32_t maxctx;
    int32_t max_len; // the launch covers contexts up to this many tokens (host argument)
    pod_bf16 *out;   // [B][Hq][D]
    // score reuse (modes 1 and 2 of the partial kernel): scaled distant logits of the block's
    // lowest layer, fp32, stored tile by tile in the register order of the S^T accumulators:
    // [B][Hkv][score_stride / (32 * rep) tiles][4 (lane / 16)][rep heads][8 tokens of the lane],
    // so that a wave writes (and later reads) 32 contiguous bytes per lane and 128 contiguous bytes
    // per 4 neighbouring lanes; preceded by a header int32 [B][Hkv][4] = (n, distant-key store of the head's block,
    // bits of the logit scale, unused)
    float *scores;
    int32_t *score_hdr;
    int32_t score_stride;
    int32_t mode;    // 0 plain; 2 score reuse; 3 score reuse with the gated skip.  With 2 and 3 a kv head for which this
                     // layer is the lowest of its block writes the logits, every other head reads them
    // gated skip of distant tokens (mode 1 writes gate_d, mode 3 uses it): per (sequence, query head)
    float *gate_d;   // [B][Hq][2]: maximum and sum of the distant exponentials at the lowest layer (base-2 domain)
    int32_t *skip;   // [B][Hq]: 1 where the upper layer left the distant part out (written by its distant pass)
    float tau;
    // merge inside the streaming kernel (FUSE >= 1): arrival counters, zero between launches.  tickets[b][kv head]
    // counts the workgroups of a (sequence, kv head) pair that have stored their partial; the last one merges.
    unsigned long long *tickets; // [max_batch][Hkv]: arrivals in bits 0-19, sum of the arrivals' XCC ids in 20-41, of their squares in 42-63
    // decode step (FUSE == 2): the new token's rows, its position, and what the cache update writes
    const u32x4 *k_new, *v_new;  // [B][Hkv][D]
    const int32_t *positions;    // [B]: position of the new token = tokens held before the call
    int32_t *lens_w;             // this layer's device-side lengths [B], advanced by the call
    int32_t *step_done;          // [max_batch]: kv heads of a sequence whose cache update is done; the last one stores the length
    int32_t low_is_self;         // lens_lowest is this layer's own array (compare it with the length before the update)
    int32_t step;                // 1: this launch is a decode step (read by decode_combine_kernel when it merges one)
    int32_t sink, window;
    // XCD-local hand-off (LOC): the launch is one-dimensional, workgroup w belongs to (sequence, kv head) pair
    // (w / nxcd / slots) * nxcd + w % nxcd
    int32_t nxcd, npairs, slots;
    // measurement aid (pod_profile_set_trace): per workgroup of a fused launch 8 words = (pair << 32 | piece, XCC id,
    // then device clock at: start, end of the tile loop, partial stored, arrival counted, end); NULL = off
    unsigned long long *trace;
    int32_t trace_cap;
    // even split (decode_even_kernel): bal_q units of kUnit tokens per workgroup (0: not this kind of launch), bal_nwg
    // workgroups that walk rows, bal_total units in all; unit_cum[b] = units of the sequences before b (per kv head)
    int32_t bal_q, bal_nwg, bal_total;
    int32_t walk_rev;            // 1: walk the tiles of the distant keys a lower layer of the block has just read from the last to the first
    int32_t bal_unit_d;          // tokens per unit of distant rows (kUnit; twice that where an upper layer reads logits instead of keys)
    int32_t hlen[kMaxHostLens];
    int32_t unit_cum[kMaxHostLens + 1];
    // per kv head: (slot * max_batch of the distant-key store the head reads at this layer) | sign bit if this
    // layer is the lowest of the head's block (then every logit of the head uses q, not q_shared)
    int32_t head_arg[kMaxKvHeads];
};
static_assert(offsetof(decode_params, hot) == 0, "hot lines first");

// The compiler places each kernel-argument load next to its first use, which turns a kernel
// prologue into a chain of dependent round trips to the argument block.  These two helpers read
// the hot line and one hlen entry with volatile scalar loads at the point of call, so both are in
// flight together before the first branch.
typedef int32_t i32x16 __attribute__((ext_vector_type(16)));
typedef int32_t i32x32 __attribute__((ext_vector_type(32)));
__device__ inline decode_hot load_hot_args()
{
    const volatile __attribute__((address_space(4))) i32x16 *ka =
        (const volatile __attribute__((address_space(4))) i32x16 *)__builtin_amdgcn_kernarg_segment_ptr();
    const i32x16 lo = ka[0], hi = ka[1];
    const i32x32 raw = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16, 17, 18, 19,
                                               20, 21, 22, 23, 24, 25, 26, 27, 28, 29, 30, 31);
    return __builtin_bit_cast(decode_hot, raw);
}
__device__ inline int load_head_arg(int h)
{
    const volatile __attribute__((address_space(4))) int32_t *ka =
        (const volatile __attribute__((address_space(4))) int32_t *)__builtin_amdgcn_kernarg_segment_ptr();
    return ka[offsetof(decode_params, head_arg) / 4 + (h < kMaxKvHeads ? h : 0)];
}
__device__ inline int load_cum_arg(int b)
{
    const volatile __attribute__((address_space(4))) int32_t *ka =
        (const volatile __attribute__((address_space(4))) int32_t *)__builtin_amdgcn_kernarg_segment_ptr();
    return ka[offsetof(decode_params, unit_cum) / 4 + (b <= kMaxHostLens ? b : 0)];
}
__device__ inline int load_hlen_arg(int b)
{
    const volatile __attribute__((address_space(4))) int32_t *ka =
        (const volatile __attribute__((address_space(4))) int32_t *)__builtin_amdgcn_kernarg_segment_ptr();
    return ka[offsetof(decode_params, hlen) / 4 + (b < kMaxHostLens ? b : 0)];
}

// Length of sequence b as validated on the device: 0 = skip (inactive, or contract violated:
// then *bad is set).  context_lens must equal the device-side length of this layer, the block's
// lowest layer must be in step once distant tokens exist, and the host mirror (which the partial
// kernel may have worked from) must agree.  The three loads are independent and issued together.
__device__ inline int decode_seq_len(const decode_params &p, int b, bool *bad)
{
    const int n = p.hot.ctx[b];
    const int dev = p.hot.lens_layer[b];
    const int low = p.hot.lens_lowest[b];
    *bad = false;
    if (n == 0) return 0;
    if (n < 0 || n > p.maxctx || n > p.max_len || n != dev || (n > p.hot.prows && low != n) || (p.hot.use_hlen && n != p.hlen[b])) {
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

// MODE 0: every logit is computed here.  MODE 1 (lowest layer of a block, score reuse): the same,
// and the scaled logits of distant chunks are also written to p.scores.  MODE 2 (upper layer, score
// reuse): distant chunks take their logits from p.scores instead of reading the block's distant
// keys (Eq. 3 line 3 says they ARE the lowest layer's logits), so such a chunk streams V only.
// Merge of np consecutive (max, sum) partials by one wave: lane l takes entries l, l + 64, ..., then a
// butterfly over the lanes; lane 0's result is broadcast so that every caller sees the same bits.
// Products and sums are explicitly rounded (no contraction): the decision derived from them must
// come out the same wherever it is evaluated.
__device__ inline float2 merged_ml(const float *ml, int np, int lane)
{
    typedef const __attribute__((address_space(1))) float *gfloat_ptr;
    float m = kNegBig, l = 0.f;
    for (int v = lane; v < np; v += 64) {
        const float m2 = ((gfloat_ptr)ml)[2 * v], l2 = ((gfloat_ptr)ml)[2 * v + 1];
        const float M = fmaxf(m, m2);
        l = __fadd_rn(__fmul_rn(l, exp2f(m - M)), __fmul_rn(l2, exp2f(m2 - M)));
        m = M;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float m2 = __shfl_xor(m, off), l2 = __shfl_xor(l, off);
        const float M = fmaxf(m, m2);
        l = __fadd_rn(__fmul_rn(l, exp2f(m - M)), __fmul_rn(l2, exp2f(m2 - M)));
        m = M;
    }
    return make_float2(__shfl(m, 0), __shfl(l, 0));
}

// g >= tau with g = P / (P + Dst), P = lp 2^mp, Dst = ld 2^md  <=>  (1 - tau) lp >= tau ld 2^(md - mp)
__device__ inline bool gate_skips(float mp, float lp, float md, float ld, float tau)
{
    if (!(ld > 0.f)) return false;  // no distant tokens: nothing to leave out
    return __fmul_rn(1.f - tau, lp) >= __fmul_rn(__fmul_rn(tau, ld), __builtin_amdgcn_exp2f(md - mp));
}

// Partials that are merged inside the same launch travel between workgroups.  The chip is 8 XCDs, each with its own L2,
// and the L2s are not coherent with each other.  Two ways to hand a partial over:
//  * LOC (the fast one): every workgroup of a (sequence, kv head) pair runs on ONE XCD - the launch is one-dimensional
//    and workgroups go to the XCDs round-robin, so the pair is chosen from (workgroup index) mod (number of XCDs).
//    Producer and consumer then meet in that XCD's L2: ordinary stores (the vector L1 writes through), an atomic
//    counter executed in the L2, ordinary loads after the consumer has dropped its own L1.  A round trip is a few
//    hundred ns.  The placement is checked, not assumed: every arrival adds the id of the XCD it runs on (XCC_ID
//    hardware register) and its square to the pair's counter word, and the merging workgroup accepts the partials
//    only if all ids were equal (n * sum of squares == square of the sum); otherwise it zeroes the output rows and
//    raises the sticky flag.  (Eager launches were seen to start their round-robin at XCD 0 and graph replays at XCD
//    7: the XCD of a position differs between launches, but a launch's workgroups of one position share it.)
//  * otherwise device-scope relaxed atomic stores (write-through: in memory when acknowledged), a device-scope atomic
//    counter and device-scope atomic loads, all of which go through to the memory fabric: correct wherever the
//    workgroups run, but ~1.6 us per round trip.  (Device-scope release/acquire FENCES are not an option here: each
//    one writes back / invalidates a whole L2, which made the launch 5x slower.)
__device__ inline int xcc_id() { return (int)(__builtin_amdgcn_s_getreg((4 - 1) << 11 | 20) & 0xf); } // HW_REG_XCC_ID[3:0]

template <bool LOC>
__device__ inline void store_part(float *p, float v)
{
    if constexpr (LOC) *(__attribute__((address_space(1))) float *)p = v;
    else __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <bool LOC, int VEC>
__device__ inline void load_part(const float *p, float (&out)[VEC])
{
    static_assert(LOC ? VEC == 4 : VEC == 2, "");
    if constexpr (LOC) {
        const f32x4 v = *(const __attribute__((address_space(1))) f32x4 *)p;
        out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
    } else {
        const unsigned long long u = __hip_atomic_load((const unsigned long long *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        out[0] = __uint_as_float((unsigned)u); out[1] = __uint_as_float((unsigned)(u >> 32));
    }
}
template <bool LOC>
__device__ inline float2 load_ml(const float *p)
{
    if constexpr (LOC) {
        typedef __attribute__((ext_vector_type(2))) float f32x2;
        const f32x2 v = *(const __attribute__((address_space(1))) f32x2 *)p;
        return make_float2(v.x, v.y);
    }
    const unsigned long long u = __hip_atomic_load((const unsigned long long *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_float2(__uint_as_float((unsigned)u), __uint_as_float((unsigned)(u >> 32)));
}

// Arrival of a workgroup whose partial is stored: returns 0 if it is not the last of `expected` arrivals; else 1 (every
// other workgroup's partial can now be read; the counter is back to zero for the next launch), or 2 if LOC and the
// arrivals did not all come from one XCD (the partials may then not be readable here).  Every thread first waits for its
// own stores to be acknowledged (by the L2 if LOC, by memory otherwise); after the barrier one thread counts, with a
// 64-bit vector atomic at device scope.
template <bool LOC>
__device__ inline int arrive_last(unsigned long long *ticket, int expected)
{
    __shared__ int sm_last;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned long long x = LOC ? (unsigned long long)xcc_id() : 0ull;
        const unsigned long long inc = 1ull | (x << 20) | ((x * x) << 42);
        const unsigned long long tot = __hip_atomic_fetch_add(ticket, inc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + inc;
        const unsigned long long n = tot & 0xfffffull, sx = (tot >> 20) & 0x3fffffull, sxx = tot >> 42;
        int last = (int)n == expected;
        if (last) {
            __hip_atomic_store(ticket, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (LOC && n * sxx != sx * sx) last = 2;
        }
        sm_last = last;
    }
    __syncthreads();
    const int last = sm_last;
    if (LOC && last) asm volatile("buffer_inv sc0" ::: "memory");   // this CU's vector L1: read the partials from the L2
    return last;
}

// MODE 3 and 4 are the two launches of a gated upper layer (appendix "Computation Optimization for Distant
// Tokens"): MODE 3 walks the proximal chunks only; MODE 4 walks the distant chunks, and each
// workgroup first evaluates the gate g = sum exp(a^P) / (sum exp(a^P) + sum exp(a^D)) of Eq. 4 for its
// query heads from the proximal partials of MODE 3 and the lowest layer's distant sums, records
// which heads have g >= tau, and leaves if all of its heads do.
template <int D, bool LOC, int NW>
__device__ void merge_and_store(const decode_params &p, const decode_hot &hot, int b, int h, int nd, int np, bool special, bool valid,
                                bool bad);
template <int D, bool LOC, int NW, int MODE>
__device__ void step_workgroup(const decode_params &p, const decode_hot &hot, int b, int h, int pos, int head_arg);

// FUSE 0: partials only, decode_combine_kernel follows.  FUSE 1 (MODE 0 only): the last workgroup of a (sequence, kv
// head) pair to store its partial merges them all and writes the output rows.  FUSE 2: FUSE 1 for a decode STEP: the
// cache holds the tokens before the new one; one workgroup of the pair (that of its last distant piece; of its first
// proximal piece where there is no distant token, and in FUSE 3) first handles the new token and the token it displaces
// from the window and performs the cache update (step_workgroup), then walks its piece like everybody else walks
// theirs: over the old rows.  FUSE 3: a step whose partials decode_combine_kernel merges
// (launches of several rounds of workgroups: there a workgroup that waits for its arrival to be counted holds its
// slot idle, which costs more than the second launch).
template <int D, int MODE, int FUSE = 0, bool LOC = false, int NW = fuse_waves(FUSE)>
__global__ __launch_bounds__(NW * 64, 8 / NW) void decode_partial_kernel(decode_params p)
{
    static_assert(FUSE == 0 || MODE == 0 || ((FUSE == 2 || FUSE == 3) && (MODE == 1 || MODE == 2)),
                  "the fused forms serve the plain mode and, as a decode step, score reuse");
    constexpr bool STEP = FUSE == 2 || FUSE == 3, MERGE = FUSE == 1 || FUSE == 2;
    static_assert(!LOC || MERGE, "the XCD-local launch shape serves the fused merge");
    constexpr int CPR = D / 8;        // 16-byte pieces per row
    constexpr int RPI = 64 / CPR;     // rows one K load instruction covers
    constexpr int NLD = kTile / RPI;  // K load instructions per tile
    constexpr int KST = D / 32;       // MFMA k-steps over the head dim
    constexpr int XN = 16 / CPR;      // lanes sharing one V piece (1 for D=128, 2 for D=64)
    constexpr int NPV = 8 / XN;       // PV MFMAs per tile

    // The arguments the first loads depend on, in one round trip to the argument block.
    const decode_hot hot = load_hot_args();
    int b = blockIdx.z, h = blockIdx.y, c = MODE == 3 ? (int)blockIdx.x + hot.max_nd : (int)blockIdx.x;
    if constexpr (LOC) {
        // one-dimensional launch: position x = w mod nxcd picks the XCD (and with it the pairs x, x + nxcd, ...), the
        // workgroups of one XCD take their pairs one after the other, each pair's pieces in order
        const int w = blockIdx.x, x = w % p.nxcd, j = w / p.nxcd;
        const int pl = j / p.slots;
        c = j - pl * p.slots;
        const int pr = pl * p.nxcd + x;
        if (pr >= p.npairs) return;
        b = pr / hot.hkv;
        h = pr - b * hot.hkv;
    }
    const int n_host = load_hlen_arg(b);
    const int head_arg = load_head_arg(h);
    // Score reuse with head-wise blocks: the writing launch (MODE 1) serves the kv heads for which this layer is
    // the lowest of the block, the reading launches (MODE 2, 3, 4) the others; with uniform blocks one of the
    // two kinds is empty and is not launched.  (Before anything else: a step's cache update belongs to one launch.)
    if (MODE == 1 && head_arg >= 0) return;
    if (MODE >= 2 && head_arg < 0) return;
    unsigned long long tr_t0 = 0, tr_t1 = 0, tr_t2 = 0;
    if (p.trace) tr_t0 = wall_clock64();
    const u32x4 *kdist = hot.kdist, *vdist = hot.vdist, *kprox = hot.kprox, *vprox = hot.vprox;
    const int cd = hot.cd, prows = hot.prows, hkv = hot.hkv, max_nd = hot.max_nd;
    const int chunk_p = (int)((unsigned)hot.chunk >> 16);
    const bool use_hlen = hot.use_hlen != 0;
    // The host mirror's length is always within the buffers; whether it agrees with context_lens
    // and the device-side lengths is checked where the partials are merged (the combine kernel or the last
    // workgroup), which zeroes the output and raises the flag if not.  Without the mirror (batches beyond
    // kMaxHostLens, or a cache set to take lengths from the device) the length comes from the call's device
    // array and is only held to the buffer and launch bounds here.
    int n = n_host;     // tokens this launch's workgroups walk (a step: the tokens held BEFORE the new one)
    if (!use_hlen) {
        if constexpr (STEP) {
            n = p.positions[b];
            if (n < 0 || n >= p.maxctx || n >= p.max_len) n = -1;
        } else if constexpr (FUSE == 1) {
            n = hot.ctx[b];
            if (n < 0 || n > p.maxctx || n > p.max_len) n = -1;
        } else {
            bool bad;
            n = decode_seq_len(p, b, &bad);
        }
    }
    if constexpr (MERGE) {
        // nothing to walk and nobody to merge: the first workgroup of the pair leaves the zeroed output rows
        // (an inactive entry), and raises the flag where the entry is not allowed to be empty
        if (n < 0 || (FUSE == 1 && n == 0)) {
            if (c == 0) {
                for (int t = threadIdx.x; t < hot.rep * (D / 2); t += blockDim.x)
                    ((unsigned *)(p.out + ((size_t)b * hot.hq + (size_t)h * hot.rep) * D))[t] = 0u;
                const bool bad = FUSE == 2 || n < 0 || hot.ctx[b] != 0;
                if (bad && h == 0 && threadIdx.x == 0) atomicOr(p.flag, 2);
            }
            return;
        }
    } else if constexpr (STEP) {
        if (n < 0) return;   // (the combine kernel zeroes the rows and raises the flag)
    } else {
        if (n <= 0) return;
    }
    const int n_prox = n < prows ? n : prows;
    const int n_dist = n - n_prox;
    // workgroups of this (sequence, kv head) pair that store a partial (FUSE >= 1): the pieces of the two regions
    // this launch's grid holds, and a step's extra workgroup
    int nd_eff = 0, np_eff = 0;
    if constexpr (MERGE) {
        nd_eff = min((n_dist + (hot.chunk & 0xffff) - 1) / (hot.chunk & 0xffff), max_nd);
        np_eff = min((n_prox + chunk_p - 1) / chunk_p, hot.nc - max_nd);
    }
    // A step: one workgroup of the pair also takes the new token and the cache update; it arrives once for both
    // partials.  FUSE 2: the workgroup of the LAST distant piece, which is the pair's shortest on average (the first
    // proximal piece, which hosted the step before, is its longest: its tile loop ended 1.35 us after the others' and
    // its pair waited for it); the first proximal piece where there is no distant token, also when the cache is empty
    // and that workgroup has no piece of its own.
    const bool hosts_step = STEP && c == (FUSE == 2 && nd_eff > 0 ? nd_eff - 1 : max_nd);
    const int expected = nd_eff + (FUSE == 2 && np_eff == 0 ? 1 : np_eff);
    if (hosts_step) step_workgroup<D, LOC, NW, MODE>(p, hot, b, h, n, head_arg);
    const bool distant = c < max_nd;
    const int region_len = distant ? n_dist : n_prox;
    const int chunk = distant ? (hot.chunk & 0xffff) : chunk_p;
    const int start = (distant ? c : c - max_nd) * chunk;
    // (a step on an empty cache: the workgroup that hosts the step walks no tile - the loads below read the region's
    // first row, which is allocated, and every position is masked - and arrives like everybody else)
    if (start >= region_len && !(FUSE == 2 && hosts_step)) return;
    const int end = min(start + chunk, region_len);
    // FUSE 2: the ring slot the new token replaces is being rewritten by step_workgroup, which also accounts for the
    // token it held: everybody else leaves that row out (its probability is forced to zero; old or new, its bytes
    // are those of a real token, so the masked products stay finite)
    const int excl = (STEP && !distant && n >= prows) ? p.sink + (n - p.sink) % p.window : -1;

    // (a step tags from the workgroup that hosts the step: the first distant piece may have no row to walk yet)
    if (MODE == 1 && (STEP ? hosts_step : c == 0) && threadIdx.x == 0) { // tag this head's logits: which token, which block's keys
        p.score_hdr[4 * ((size_t)b * hkv + h)] = STEP ? n + 1 : n;   // (the context the attention is over)
        p.score_hdr[4 * ((size_t)b * hkv + h) + 1] = head_arg & 0x7fffffff;
        p.score_hdr[4 * ((size_t)b * hkv + h) + 2] = __float_as_int(hot.scale_log2e);
        // word 3: 1 once the heads' distant (maximum, sum) pairs are there too (decode_combine_kernel leaves them after a
        // pod_decode_attention_reuse / _gated call; a step and the merge inside the launch do not), which is what a
        // gated upper layer needs besides the logits
        if (MERGE || STEP) p.score_hdr[4 * ((size_t)b * hkv + h) + 3] = 0;
    }
    // (pointers rebuilt from the raw argument words are generic; say they are global memory)
    typedef const __attribute__((address_space(1))) u32x4 *gvec_ptr;
    const size_t pair = (size_t)b * hkv + h;
    const size_t kslot_row = (size_t)(head_arg & 0x7fffffff) + b; // distant keys live per (kv head, block): [slot][B][cd]
    const gvec_ptr Kb = (gvec_ptr)(distant ? kdist + kslot_row * cd * CPR : kprox + pair * prows * CPR);
    const gvec_ptr Vb = (gvec_ptr)(distant ? vdist + pair * cd * CPR : vprox + pair * prows * CPR);
    const pod_bf16 *qsrc = (distant && hot.q_shared && head_arg >= 0) ? hot.q_shared : hot.q;

    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int m16 = lane & 15, j = lane >> 4;

    // NW K tiles of kTile rows; the same bytes later hold the merge buffer [NW][rep <= 16][RS] floats.  Its rows are
    // padded (4 floats after every 32 dims, row stride 1 mod 32): the 16 lanes of a wave that hold real heads write
    // the same (i, x) element of 4 heads x 4 dim groups at once, which would otherwise all fall into one LDS bank.
    constexpr int RS = D + 4 * (D / 32) + 1;
    constexpr size_t kTileBytes = sizeof(u32x4) * NW * kTile * CPR, kMergeBytes = sizeof(float) * NW * 16 * RS;
    __shared__ __attribute__((aligned(16))) char lds_raw[kTileBytes > kMergeBytes ? kTileBytes : kMergeBytes];
    u32x4 *ldsK = (u32x4 *)lds_raw + (size_t)wave * kTile * CPR;

    f32x4 acc[NPV];
#pragma unroll
    for (int x = 0; x < NPV; ++x) acc[x] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = kNegBig, l_run = 0.f;

    const int kr = lane / CPR, kc = lane % CPR; // K load: row within the instruction, piece
    const int vc = lane % CPR;                  // V load: piece
    const int vx = (lane / CPR) % XN;           // which of the XN dims per piece pair this lane serves
    const int last = end > 0 ? end - 1 : 0;

    // Tile loads.  Rows of a tile past the chunk's end are clamped to its last row (valid memory, masked later), so
    // a tile's loads need no per-lane branches; whole tiles past the end are not requested (a wave-uniform test).
    // V is read non-temporally, K with ordinary loads: every row is used once per launch, and a stream that does not
    // settle in the L2 leaves the partials, the queries and the other stream alone.  Measured, whole decode steps
    // (one sequence of 32K tokens in us; 16 ragged sequences and 4 x 128K tokens in ms; plain / score reuse):
    //   both ordinary 58.9 / 67.6, 6.88 / 6.23, 11.94 / 8.68      V non-temporal 56.3 / 64.4, 6.28 / 5.91, 10.83 / 7.98
    //   K non-temporal 60.1 / 66.3, 6.28 / 6.04, 10.82 / 8.46     both           57.6 / 62.7, 6.21 / 5.89, 11.01 / 8.06
    u32x4 kreg[NLD], vreg[8];
#define POD_LOAD_TILE(T0)                                                         \
    _Pragma("unroll") for (int i = 0; i < NLD; ++i) {                             \
        const int row = min((T0) + RPI * i + kr, last);                           \
        kreg[i] = Kb[(size_t)row * CPR + kc];                                     \
    }                                                                             \
    _Pragma("unroll") for (int e = 0; e < 8; ++e) {                               \
        const int tok = (e < 4) ? 4 * j + e : 16 + 4 * j + (e - 4);               \
        const int row = min((T0) + tok, last);                                    \
        vreg[e] = __builtin_nontemporal_load(&Vb[(size_t)row * CPR + vc]);        \
    }

    int t0 = start + wave * kTile;
    const bool reads_scores = (MODE == 2 || MODE == 4) && distant; // such a chunk needs neither K nor Q
    if constexpr (MODE == 4) {
        if (!distant) return;
        // ---- the gate of this workgroup's heads: every wave computes the same values, 16 lanes per
        // head (four heads at a time), all loads of a pass in flight together
        typedef const __attribute__((address_space(1))) float *gfloat_ptr;
        const int np = (n_prox + chunk_p - 1) / chunk_p;
        const int sub = lane & 15, grp = lane >> 4;
        bool all_skip = true;
        for (int h0 = 0; h0 < hot.rep; h0 += 4) {
            const int hh = min(h0 + grp, hot.rep - 1);     // (a group past the last head repeats it)
            const int head = h * hot.rep + hh;
            const gfloat_ptr ml = (gfloat_ptr)(hot.part_ml + ((size_t)b * hot.hq + head) * hot.nc * 2 + (size_t)max_nd * 2);
            const gfloat_ptr gd = (gfloat_ptr)(p.gate_d + ((size_t)b * hot.hq + head) * 2);
            const float md = gd[0], ld = gd[1];
            float m = kNegBig, l = 0.f;
            for (int v = sub; v < np; v += 16) {
                const float m2 = ml[2 * v], l2 = ml[2 * v + 1];
                const float M = fmaxf(m, m2);
                l = __fadd_rn(__fmul_rn(l, __builtin_amdgcn_exp2f(m - M)), __fmul_rn(l2, __builtin_amdgcn_exp2f(m2 - M)));
                m = M;
            }
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) {
                const float m2 = __shfl_xor(m, off), l2 = __shfl_xor(l, off);
                const float M = fmaxf(m, m2);
                l = __fadd_rn(__fmul_rn(l, __builtin_amdgcn_exp2f(m - M)), __fmul_rn(l2, __builtin_amdgcn_exp2f(m2 - M)));
                m = M;
            }
            m = __shfl(m, lane & 48);                      // the group's first lane decides for all
            l = __shfl(l, lane & 48);
            const bool sk = gate_skips(m, l, md, ld, p.tau);
            all_skip = all_skip && __all(sk);
            if (c == 0 && wave == 0 && sub == 0 && h0 + grp < hot.rep) p.skip[(size_t)b * hot.hq + head] = sk ? 1 : 0;
        }
        if (all_skip) return;
    }
    // The wave's tiles, first + k NW kTile below `end`.  Every second layer of a block walks its distant tiles from the last
    // to the first: the layer below has just read the same keys (one launch earlier, same pieces, same XCD), and what of
    // them is still in that XCD's L2 are the tiles it read last (config 2: 56.6 -> 55.6 us per step).
    const int first = t0;
    const int ntile_w = first < end ? (end - first + NW * kTile - 1) / (NW * kTile) : 0;
    const bool rev = p.walk_rev != 0 && !reads_scores && distant && head_arg >= 0;
    const int tstep = rev ? -(NW * kTile) : NW * kTile;
    if (rev && ntile_w > 0) t0 = first + (ntile_w - 1) * (NW * kTile);
    if (!reads_scores && ntile_w > 0) { POD_LOAD_TILE(t0) }

    // Q as B operand: lane (head m16, j) holds dims 32s + 8j .. +7 of its head (zero past rep).
    bf16x8 qf[KST];
    {
        const gvec_ptr qrow = (gvec_ptr)(qsrc + ((size_t)b * hot.hq + (size_t)h * hot.rep + m16) * D);
#pragma unroll
        for (int s = 0; s < KST; ++s) {
            u32x4 t = u32x4{0u, 0u, 0u, 0u};
            if (m16 < hot.rep && !reads_scores) t = qrow[4 * s + j];
            qf[s] = as_bf16x8(t);
        }
    }


    // ---- online softmax for head m16 over this lane's 8 tokens (base-2 domain), then O^T += V^T P
    auto softmax_pv = [&](float (&sc)[8], const u32x4 (&vcur)[8]) {
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
    };

    if (reads_scores) {
        // Score reuse: this chunk's logits were written by the block's lowest layer (already scaled,
        // base-2 domain) in exactly the per-lane order of the S^T accumulators: head m16, tokens
        // 4j..4j+3 of the two 16-token halves of a tile.  Only V is streamed.
        typedef const __attribute__((address_space(1))) f32x4 *gf4_r;
        const gf4_r sbase = (gf4_r)(p.scores + ((size_t)b * hkv + h) * p.score_stride * hot.rep) +
                            ((size_t)j * hot.rep + (m16 < hot.rep ? m16 : 0)) * 2;
        // Half the bytes per token means half the bytes in flight per wave, so two tiles are kept
        // in flight here (register sets A and B) instead of one.
        f32x4 sregA[2], sregB[2];
        u32x4 vregB[8];
#define POD_LOAD_SV(SR, VR, T0)                                                   \
        {                                                                             \
            const gf4_r sp = sbase + (size_t)(min((T0), last) >> 5) * 8 * hot.rep;     \
            SR[0] = sp[0];                                                            \
            SR[1] = sp[1];                                                            \
        }                                                                             \
        _Pragma("unroll") for (int e = 0; e < 8; ++e) {                               \
            const int tok = (e < 4) ? 4 * j + e : 16 + 4 * j + (e - 4);               \
            const int row = min((T0) + tok, last);                                    \
            VR[e] = __builtin_nontemporal_load(&Vb[(size_t)row * CPR + vc]);          \
        }
#define POD_CONSUME_SV(SR, VR, T0, TNEXT)                                         \
        {                                                                             \
            u32x4 vcur[8];                                                            \
            float sc[8];                                                              \
            _Pragma("unroll") for (int e = 0; e < 8; ++e) vcur[e] = VR[e];            \
            _Pragma("unroll") for (int i = 0; i < 4; ++i) {                           \
                const int tok0 = (T0) + 4 * j + i, tok1 = tok0 + 16;                  \
                sc[i] = tok0 < end ? SR[0][i] : kNegBig;                              \
                sc[4 + i] = tok1 < end ? SR[1][i] : kNegBig;                          \
            }                                                                         \
            if (m16 >= hot.rep) {                                                     \
                _Pragma("unroll") for (int i = 0; i < 8; ++i) sc[i] = 0.f; /* padding heads: any finite value */ \
            }                                                                         \
            if ((TNEXT) < end) { POD_LOAD_SV(SR, VR, TNEXT) } /* (never past the piece: see the K/V loop) */ \
            softmax_pv(sc, vcur);                                                     \
        }
        constexpr int kStep = NW * kTile;
        if (t0 < end) { POD_LOAD_SV(sregA, vreg, t0) }
        if (t0 + kStep < end) { POD_LOAD_SV(sregB, vregB, t0 + kStep) }
        for (; t0 < end; t0 += 2 * kStep) {
            POD_CONSUME_SV(sregA, vreg, t0, t0 + 2 * kStep)
            if (t0 + kStep < end) POD_CONSUME_SV(sregB, vregB, t0 + kStep, t0 + 3 * kStep)
        }
#undef POD_CONSUME_SV
#undef POD_LOAD_SV
    } else
    for (int it = 0; it < ntile_w; ++it, t0 += tstep) {
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

        // ---- next tile's loads go out before the softmax / PV work of this one.  Not past the piece's end: nothing
        // would use them, and the wave would still wait for them before it may hand its partial over and end (as long
        // as any other load on a saturated memory system: 3 us per workgroup measured).
        if (it + 1 < ntile_w) { POD_LOAD_TILE(t0 + tstep) }

        // ---- online softmax for head m16 over this lane's 8 tokens (base-2 domain)
        float sc[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int tok0 = t0 + 4 * j + i, tok1 = tok0 + 16;
            sc[i] = (tok0 < end && (!STEP || tok0 != excl)) ? s0[i] * hot.scale_log2e : kNegBig;
            sc[4 + i] = (tok1 < end && (!STEP || tok1 != excl)) ? s1[i] * hot.scale_log2e : kNegBig;
        }
        if constexpr (MODE == 1) {
            if (distant && m16 < hot.rep) { // the lowest layer's distant logits, for the block's upper layers
                typedef __attribute__((address_space(1))) f32x4 *gf4_w;
                const size_t tile = (size_t)(t0 >> 5);
                const gf4_w dst = (gf4_w)(p.scores + ((size_t)b * hkv + h) * p.score_stride * hot.rep) +
                                  (tile * 4 * hot.rep + (size_t)j * hot.rep + m16) * 2;
                if (!STEP || t0 + kTile <= end) {
                    // (tokens past the chunk carry the mask value.  Non-temporal stores: stores inside the read stream cost
                    // far more than their bytes - a layer that writes logits takes 17-22 % longer for 3 % more bytes - and
                    // lines that do not settle in the L2 cost a little less: score-reuse steps 1-2 % faster)
                    __builtin_nontemporal_store(f32x4{sc[0], sc[1], sc[2], sc[3]}, &dst[0]);
                    __builtin_nontemporal_store(f32x4{sc[4], sc[5], sc[6], sc[7]}, &dst[1]);
                } else {   // a step's last, partly filled tile: the element behind the last row is step_workgroup's to store
                    typedef __attribute__((address_space(1))) float *gf_w;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if (t0 + 4 * j + i < end) ((gf_w)dst)[i] = sc[i];
                        if (t0 + 16 + 4 * j + i < end) ((gf_w)dst)[4 + i] = sc[4 + i];
                    }
                }
            }
        }
        softmax_pv(sc, vcur);
    }

#undef POD_LOAD_TILE
    // ---- merge the waves of this workgroup, write one partial per (head, chunk)
    // acc[x][i] is O^T[dim slot 4j+i][head m16]; the slot's dim is
    //   XN = 1: 8*(4j+i) + x        XN = 2: 8*((4j+i) % 8) + 2x + (4j+i)/8
    __syncthreads(); // all waves are done with their K tiles
    if (p.trace) tr_t1 = wall_clock64();
    float *sm_acc = (float *)lds_raw;                 // [NW][rep][RS], dim d of a row at d + 4 (d / 32)
    __shared__ float sm_m[NW][16], sm_l[NW][16];
    if (m16 < hot.rep) {
#pragma unroll
        for (int x = 0; x < NPV; ++x)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int slot = 4 * j + i;
                const int dim = (XN == 1) ? 8 * slot + x : 8 * (slot % 8) + 2 * x + slot / 8;
                sm_acc[((size_t)wave * hot.rep + m16) * RS + dim + 4 * (dim >> 5)] = acc[x][i];
            }
        if (j == 0) { sm_m[wave][m16] = m_run; sm_l[wave][m16] = l_run; }
    }
    __syncthreads();
    const int NC = hot.nc + (STEP ? 1 : 0); // (a step keeps one more slot per head: step_workgroup's)
    for (int t = threadIdx.x; t < hot.rep * D; t += blockDim.x) {
        const int head = t / D, dim = t % D;
        float M = sm_m[0][head];
#pragma unroll
        for (int w = 1; w < NW; ++w) M = fmaxf(M, sm_m[w][head]);
        float A = 0.f, Lsum = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float f = exp2f(sm_m[w][head] - M);
            A += f * sm_acc[((size_t)w * hot.rep + head) * RS + dim + 4 * (dim >> 5)];
            Lsum += f * sm_l[w][head];
        }
        typedef __attribute__((address_space(1))) float *gfloat_ptr;
        // (merged inside the launch: a sequence's pieces stand one after the other, its proximal ones right behind its
        // distant ones, so that the merging workgroup addresses them by one stride)
        const size_t slot = ((size_t)b * hot.hq + (size_t)h * hot.rep + head) * NC + (MERGE && !distant ? nd_eff + (c - max_nd) : c);
        if constexpr (MERGE) {   // read by another workgroup of this launch
            store_part<LOC>(hot.part_acc + slot * D + dim, A);
            if (dim == 0) { store_part<LOC>(hot.part_ml + slot * 2, M); store_part<LOC>(hot.part_ml + slot * 2 + 1, Lsum); }
        } else {
            ((gfloat_ptr)hot.part_acc)[slot * D + dim] = A;
            if (dim == 0) { ((gfloat_ptr)hot.part_ml)[slot * 2] = M; ((gfloat_ptr)hot.part_ml)[slot * 2 + 1] = Lsum; }
        }
    }
    if constexpr (!MERGE) {
        const size_t wg = ((size_t)b * hkv + h) * hot.nc + c;
        if (p.trace && threadIdx.x == 0 && wg < (size_t)p.trace_cap) {
            unsigned long long *t = p.trace + 8 * wg;
            t[0] = ((unsigned long long)(b * hkv + h) << 32) | (unsigned)c;
            t[1] = (unsigned long long)xcc_id() | ((unsigned long long)__builtin_amdgcn_s_getreg((32 - 1) << 11 | 4) << 8);
            t[2] = tr_t0; t[3] = tr_t1; t[6] = wall_clock64();
        }
    }
    if constexpr (MERGE) {
        if (p.trace) tr_t2 = wall_clock64();
        const int last = arrive_last<LOC>(p.tickets + (size_t)b * hkv + h, expected);
        const unsigned long long tr_t3 = p.trace ? wall_clock64() : 0;
        auto trace_out = [&]() {
            const size_t wg = LOC ? (size_t)blockIdx.x : ((size_t)b * hkv + h) * hot.nc + c;
            if (p.trace && threadIdx.x == 0 && wg < (size_t)p.trace_cap) {
                unsigned long long *t = p.trace + 8 * wg;
                t[0] = ((unsigned long long)(b * hkv + h) << 32) | (unsigned)c | (last ? 0x80000000u : 0u);
                t[1] = (unsigned long long)xcc_id();
                t[2] = tr_t0; t[3] = tr_t1; t[4] = tr_t2; t[5] = tr_t3; t[6] = wall_clock64();
            }
        };
        if (!last) { trace_out(); return; }
        bool valid = last == 1, bad = last == 2;
        if (bad && threadIdx.x == 0) atomicOr(p.flag, 4);
        if constexpr (FUSE == 1) { // the same rule as decode_seq_len, with the host mirror's length where the walk used it
            const int v_ctx = hot.ctx[b], v_dev = hot.lens_layer[b], v_low = hot.lens_lowest[b];
            if (v_ctx == 0) valid = false;
            else if (!valid) {}
            else if (v_ctx < 0 || v_ctx > p.maxctx || v_ctx > p.max_len || v_ctx != v_dev || (v_ctx > prows && v_low != v_ctx) || v_ctx != n) {
                valid = false; bad = true;
            }
        }
        if constexpr (MODE == 2) { // the distant logits must be those of this token and of the head's block
            const size_t tag = 4 * ((size_t)b * hkv + h);
            const int n_ctx = STEP ? n + 1 : n;
            if (n_ctx > prows && (p.score_hdr[tag] != n_ctx || p.score_hdr[tag + 1] != (head_arg & 0x7fffffff) ||
                                  p.score_hdr[tag + 2] != __float_as_int(hot.scale_log2e))) {
                valid = false; bad = true;
            }
        }
        merge_and_store<D, LOC, NW>(p, hot, b, h, nd_eff, np_eff, FUSE == 2, valid, bad);
        trace_out();
    }
}

// Reductions over the 64 lanes of a wave without LDS round trips (a cross-lane read through LDS takes about 60 ns,
// and a reduction is a chain of six): four DPP steps inside the rows of 16 lanes, then the four rows through SGPRs.
// Call with all lanes active.
template <int CTRL>
__device__ inline float dpp_move(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
__device__ inline float lane_value(float v, int lane) { return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane)); }
__device__ inline float wave_max(float v)
{
    v = fmaxf(v, dpp_move<0xB1>(v));    // quad_perm [1, 0, 3, 2]
    v = fmaxf(v, dpp_move<0x4E>(v));    // quad_perm [2, 3, 0, 1]
    v = fmaxf(v, dpp_move<0x141>(v));   // row_half_mirror
    v = fmaxf(v, dpp_move<0x140>(v));   // row_mirror
    return fmaxf(fmaxf(lane_value(v, 0), lane_value(v, 16)), fmaxf(lane_value(v, 32), lane_value(v, 48)));
}
__device__ inline float wave_sum(float v)
{
    v += dpp_move<0xB1>(v);
    v += dpp_move<0x4E>(v);
    v += dpp_move<0x141>(v);
    v += dpp_move<0x140>(v);
    return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}

// The merge of a (sequence, kv head) pair's partials by the last workgroup to arrive: the same merge as
// decode_combine_kernel (the paper's gate, Eq. 4, applied to unnormalised sums).  Its time is the time of one CU's
// loads, so as many waves as possible take part and every load of a wave is in flight before the first is used:
// a query head goes to SPLIT waves (2 where the workgroup has at least two waves per head), wave s of them takes the
// partials s, s + SPLIT, ...; lane i of a wave takes the (maximum, normaliser) pair of the wave's i-th partial, each
// of the wave's 64 / LPR lane groups every NGW-th of the wave's rows, VEC floats per lane, CAP rows per lane group at
// a time (more only in launches with more than CAP * NGW * SPLIT pieces per pair: then by a running maximum).
// Maximum and normaliser are reduced over the wave, each lane computes the weight of its own partial once, and the row
// weights reach the lane groups through SGPRs; the waves of a head meet in LDS.
// nd, np: distant and proximal pieces that stored a partial; special: a step's extra partial in slot hot.nc, whose
// normaliser is negative if the step's validation failed; it is the state the head's first wave starts from.
// Called by every thread of the workgroup.
template <int D, bool LOC, int NW, int SPLIT>
__device__ void merge_and_store_split(const decode_params &p, const decode_hot &hot, int b, int h, int nd, int np, bool special, bool valid,
                                      bool bad)
{
    constexpr int VEC = LOC ? 4 : 2, LPR = D / VEC, NGW = 64 / LPR, CAP = 32 / NGW, ROWS = CAP * NGW;   // ROWS = 32 per wave
    constexpr unsigned ROWB = D * sizeof(float);
    __shared__ float sm_a[NW][D], sm_ml[NW][2];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, x = lane % LPR, g = lane / LPR;
    const int nv = nd + np;         // the pieces' partials are rows 0 .. nv - 1 of a head's block, the step's is row hot.nc
    const size_t stride = (size_t)hot.nc + (special ? 1 : 0);
    constexpr int split = SPLIT, heads_at_once = NW / split;
    for (int r0 = 0; r0 < hot.rep; r0 += heads_at_once) {
        const int r = r0 + wave / split, s = wave % split;
        const bool active = r < hot.rep;
        const int head = h * hot.rep + (active ? r : 0);
        // (wave-uniform bases and 32-bit lane offsets: the address arithmetic stands between the arrival and the first
        // load, so it is kept to two or three instructions per load)
        const char *ml = (const char *)(hot.part_ml + ((size_t)b * hot.hq + head) * stride * 2);
        const char *pa = (const char *)(hot.part_acc + ((size_t)b * hot.hq + head) * stride * D);
        float m_run = kNegBig, L = 0.f, a[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) a[e] = 0.f;
        if (active) {
            float2 mark = make_float2(kNegBig, 0.f);
            float as[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) as[e] = 0.f;
            const bool mine = special && s == 0;
            if (mine) {
                mark = load_ml<LOC>((const float *)(ml + (unsigned)hot.nc * 8u));
                load_part<LOC, VEC>((const float *)(pa + ((unsigned)hot.nc * ROWB + VEC * 4u * x)), as);
            }
            // this wave's i-th row of a block starting at v0 is partial v0 + i * split + s; lane group g takes its
            // rows g, g + NGW, ...
            constexpr unsigned kstride = (unsigned)(NGW * split) * ROWB;
            for (int v0 = 0; v0 == 0 || v0 + s < nv; v0 += ROWS * split) {
                const int first = v0 + s;
                const int vl = first + lane * split;
                const bool have = lane < ROWS && vl < nv;
                float2 mk = make_float2(kNegBig, 0.f);
                if (have) mk = load_ml<LOC>((const float *)(ml + (unsigned)vl * 8u));
                // rows past the end read the lane group's last valid row (or the wave's first) and get weight 0
                const int gfirst = first + g * split;
                int cnt = gfirst < nv ? (nv - gfirst + NGW * split - 1) / (NGW * split) : 0;
                cnt = cnt < CAP ? cnt : CAP;
                const unsigned off0 = (unsigned)gfirst * ROWB + VEC * 4u * x;
                const unsigned off_last = cnt > 0 ? off0 + (unsigned)(cnt - 1) * kstride : (unsigned)first * ROWB + VEC * 4u * x;
                float ak[CAP][VEC];
#pragma unroll
                for (int k = 0; k < CAP; ++k) {
                    const unsigned off = off0 + (unsigned)k * kstride;
                    // (wave-uniform: whole instructions past the end are not issued)
                    if (first + k * NGW * split < nv) load_part<LOC, VEC>((const float *)(pa + (off < off_last ? off : off_last)), ak[k]);
                    else
#pragma unroll
                        for (int e = 0; e < VEC; ++e) ak[k][e] = 0.f;
                }
                if (v0 == 0 && mine) {     // (loaded above, so that its latency overlaps the block's)
                    if (mark.y < 0.f) { valid = false; bad = true; }
                    m_run = mark.x; L = mark.y;
#pragma unroll
                    for (int e = 0; e < VEC; ++e) a[e] = g == 0 ? as[e] : 0.f;
                }
                const float m_new = fmaxf(m_run, wave_max(mk.x));
                const float alpha = exp2f(m_run - m_new);
                const float w = have ? exp2f(mk.x - m_new) : 0.f;
                L = L * alpha + wave_sum(w * mk.y);
#pragma unroll
                for (int e = 0; e < VEC; ++e) a[e] *= alpha;
#pragma unroll
                for (int k = 0; k < CAP; ++k) {
                    if (first + k * NGW * split < nv) {       // (wave-uniform; rows past the end were not loaded)
                        float f = lane_value(w, k * NGW);     // the weight of this lane group's k-th row
#pragma unroll
                        for (int gg = 1; gg < NGW; ++gg) f = g == gg ? lane_value(w, k * NGW + gg) : f;
#pragma unroll
                        for (int e = 0; e < VEC; ++e) a[e] += f * ak[k][e];
                    }
                }
                m_run = m_new;
            }
#pragma unroll
            for (int off = LPR; off < 64; off <<= 1)     // the lane groups of the wave (one maximum for all of them)
#pragma unroll
                for (int e = 0; e < VEC; ++e) a[e] += __shfl_xor(a[e], off);
        }
        if (split == 2) {                                // the head's second wave hands its sums to the first
            if (active && s == 1) {
                if (g == 0)
#pragma unroll
                    for (int e = 0; e < VEC; ++e) sm_a[wave][VEC * x + e] = a[e];
                if (lane == 0) { sm_ml[wave][0] = m_run; sm_ml[wave][1] = L; }
            }
            __syncthreads();
            if (active && s == 0) {
                const float m2 = sm_ml[wave + 1][0], L2 = sm_ml[wave + 1][1];
                const float m_new = fmaxf(m_run, m2);
                const float f1 = exp2f(m_run - m_new), f2 = exp2f(m2 - m_new);
                L = f1 * L + f2 * L2;
#pragma unroll
                for (int e = 0; e < VEC; ++e) a[e] = f1 * a[e] + f2 * sm_a[wave + 1][VEC * x + e];
            }
            if (r0 + heads_at_once < hot.rep) __syncthreads();   // (before the next round writes the buffer again)
        }
        if (active && s == 0 && g == 0) {
            unsigned res[VEC / 2];
#pragma unroll
            for (int e = 0; e < VEC / 2; ++e) res[e] = 0u;
            if (valid) {
                const float inv = 1.f / L;
#pragma unroll
                for (int e = 0; e < VEC / 2; ++e) res[e] = pack_bf16(a[2 * e] * inv, a[2 * e + 1] * inv);
            }
            unsigned *dst = (unsigned *)(p.out + ((size_t)b * hot.hq + head) * D) + (VEC / 2) * x;
#pragma unroll
            for (int e = 0; e < VEC / 2; ++e) dst[e] = res[e];
        }
    }
    if (bad && threadIdx.x == 0) atomicOr(p.flag, 2);
}
template <int D, bool LOC, int NW>
__device__ void merge_and_store(const decode_params &p, const decode_hot &hot, int b, int h, int nd, int np, bool special, bool valid,
                                bool bad)
{
    if (hot.rep * 2 <= NW) merge_and_store_split<D, LOC, NW, 2>(p, hot, b, h, nd, np, special, valid, bad);
    else merge_and_store_split<D, LOC, NW, 1>(p, hot, b, h, nd, np, special, valid, bad);
}

__device__ inline float dot8_bf16(u32x4 a, u32x4 b)
{
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        s = fmaf(__uint_as_float(a[w] << 16), __uint_as_float(b[w] << 16), s);
        s = fmaf(__uint_as_float(a[w] & 0xffff0000u), __uint_as_float(b[w] & 0xffff0000u), s);
    }
    return s;
}

// A decode step's extra work for one (sequence, kv head) pair, done by one of the pair's workgroups (the even split:
// by a workgroup of its own) before it turns to its piece: the new token at position pos and, once the
// window is full, the token at pos - W that it displaces (derived from the index ranges of Eq. 3: that token turns
// distant).  It (1) checks the position against the stored length, (2) stores a partial over these two tokens - the
// new one proximal, with the layer's own query and the new key; the displaced one distant, with the key the block's
// lowest layer holds for it and that layer's query - taking the displaced token's value and (at a lowest layer) key
// from the ring slot before (3) it overwrites that slot with the new rows and moves the old ones to the distant
// stores, exactly as the append kernel does.  Nobody else in the launch reads or writes those rows' results: the other
// workgroups walk the rows held before the call and leave the ring slot out.  (4) The last of a sequence's kv heads
// to finish advances the stored length; (5) the partial (in the slot behind the pieces' slots) takes part in the merge
// like any other.
// With score reuse (MODE 1: this layer is the lowest of the block; MODE 2: an upper layer) the displaced token's
// distant logit is computed once, by the lowest layer, which stores it at that token's place in the score tiles (the
// workgroups that walk the rows held before the call leave that place alone); the block's upper layers read it there.
template <int D, bool LOC, int NW, int MODE>
__device__ void step_workgroup(const decode_params &p, const decode_hot &hot, int b, int h, int pos, int head_arg)
{
    constexpr int CPR = D / 8;
    typedef const __attribute__((address_space(1))) u32x4 *gvec_ptr;
    typedef __attribute__((address_space(1))) u32x4 *gvec_w;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int prows = hot.prows;
    const int v_pos = p.positions[b], v_dev = hot.lens_layer[b], v_low = hot.lens_lowest[b];
    const bool demote = pos >= prows;           // the ring is full: its slot holds position pos - W
    bool ok = v_pos == pos && v_dev == pos && pos < p.maxctx && pos < p.max_len;
    if (demote && !p.low_is_self && v_low != pos + 1) ok = false;   // the block's lowest layer took this token first
    const int slot = pos < p.sink ? pos : p.sink + (pos - p.sink) % p.window;
    const size_t pair = (size_t)b * hot.hkv + h;
    const bool low_head = head_arg < 0;
    const size_t t = demote ? (size_t)(pos - prows) : 0;   // distant row of position pos - W
    const gvec_w proxK = (gvec_w)(hot.kprox + (pair * prows + slot) * CPR), proxV = (gvec_w)(hot.vprox + (pair * prows + slot) * CPR);
    const gvec_w dV = (gvec_w)(hot.vdist + (pair * hot.cd + t) * CPR);
    const gvec_w dK = (gvec_w)(hot.kdist + (((size_t)(head_arg & 0x7fffffff) + b) * hot.cd + t) * CPR);
    const int i = lane < CPR ? lane : 0;        // this lane's 16-byte piece of a row
    const u32x4 kn = ((gvec_ptr)p.k_new)[pair * CPR + i], vn = ((gvec_ptr)p.v_new)[pair * CPR + i];
    u32x4 ko = {0u, 0u, 0u, 0u}, vo = ko, kd = ko;
    if (demote) {
        ko = proxK[i];
        vo = proxV[i];
        if (MODE != 2) kd = low_head ? ko : dK[i];
    }
    const pod_bf16 *qd_src = (hot.q_shared && !low_head) ? hot.q_shared : hot.q;
    const size_t stride = (size_t)hot.nc + 1;
    for (int r = wave; r < hot.rep; r += NW) {
        const size_t head = (size_t)b * hot.hq + (size_t)h * hot.rep + r;
        const u32x4 qn = ((gvec_ptr)(hot.q + head * D))[i], qd = ((gvec_ptr)(qd_src + head * D))[i];
        float sn = lane < CPR ? dot8_bf16(qn, kn) : 0.f, sd = (MODE != 2 && lane < CPR && demote) ? dot8_bf16(qd, kd) : 0.f;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) { sn += __shfl_xor(sn, off); sd += __shfl_xor(sd, off); }
        sn *= hot.scale_log2e;
        sd = demote ? sd * hot.scale_log2e : kNegBig;
        if constexpr (MODE == 1 || MODE == 2) {
            if (demote) {   // distant row t of the score tiles: tile t / 32, element (lane group j, half, i) of query head r
                const int tok = (int)(t & 31);
                float *slot = p.scores + pair * p.score_stride * hot.rep +
                              ((((t >> 5) * 4 + ((tok & 15) >> 2)) * hot.rep + r) * 2 + (tok >> 4)) * 4 + (tok & 3);
                if (MODE == 1) { if (lane == 0) *slot = sd; }
                else sd = *slot;
            }
        }
        const float m = fmaxf(sn, sd);
        const float pn = exp2f(sn - m), pd = demote ? exp2f(sd - m) : 0.f;
        const size_t ps = head * stride + hot.nc;
        if (lane < CPR) {
            float *dst = hot.part_acc + ps * D + 8 * lane;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                store_part<LOC>(dst + 2 * w, pn * __uint_as_float(vn[w] << 16) + pd * __uint_as_float(vo[w] << 16));
                store_part<LOC>(dst + 2 * w + 1, pn * __uint_as_float(vn[w] & 0xffff0000u) + pd * __uint_as_float(vo[w] & 0xffff0000u));
            }
        }
        if (lane == 0) {
            store_part<LOC>(hot.part_ml + ps * 2, m);
            store_part<LOC>(hot.part_ml + ps * 2 + 1, ok ? pn + pd : -1.f);
        }
    }
    __syncthreads(); // every wave holds the old rows it needs
    if (ok && wave == 0 && lane < CPR) {
        if (demote) {
            dV[lane] = vo;
            if (low_head) dK[lane] = ko;
        }
        proxK[lane] = kn;
        proxV[lane] = vn;
    }
    // every kv head's workgroup has compared the position with the stored length before the length moves
    // (a sequence's kv heads run on different XCDs; nothing but the count travels through this counter, and nobody
    // waits for it; by this barrier every wave has used the stored length it loaded)
    __syncthreads();
    if (threadIdx.x == 0) {
        const int old = __hip_atomic_fetch_add(p.step_done + b, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old == hot.hkv - 1) {
            __hip_atomic_store(p.step_done + b, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (ok) p.lens_w[b] = pos + 1;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Launches of several rounds of workgroups (large batches, long contexts): the even split.  MODE 0: plain.  MODE 2: the
// decode step of an upper layer with score reuse (distant rows: values and the lowest layer's logits, no keys).
//
// With one piece of a fixed number of tokens per workgroup such a launch ends with a round that is partly empty, and
// every workgroup pays its start and its hand-over (measured at 16 ragged sequences: 188 us where the same bytes take a
// plain read 166 us; 4 x 128K tokens: 319-330 against 302).  Here the launch is ONE round: two workgroups per CU, and
// each walks the same number of rows.  All rows of the batch stand in one line - sequence after sequence, inside a
// sequence kv head after kv head, inside a (sequence, kv head) pair its distant rows, then its proximal rows - counted
// in units of kUnit tokens (a region's last unit may be short).  Workgroup w takes units [w q, (w + 1) q).  Where its
// part crosses from one pair into the next it hands a partial over and starts afresh; where it crosses from a pair's
// distant rows into its proximal rows it only switches operands (the softmax runs over both, Eq. 3).  A pair's
// partials come from consecutive workgroups w_lo .. w_hi and sit in its slots 0 .. w_hi - w_lo; decode_combine_kernel
// works the same numbers out from the lengths.  The lengths are the host mirror's (kernel arguments): without a
// mirror the launch keeps to fixed pieces.  STEP: bal_nwg more workgroups follow, one per pair, for the new token and
// the cache update (step_workgroup); the others leave the ring slot it rewrites out, as in decode_partial_kernel.
// The tile loops are decode_partial_kernel's: the plain one, and for MODE 2's distant rows the one that reads logits;
// there a unit of distant rows is twice as many tokens (even_unit_distant), so that all units cost about the same.
template <int D, bool STEP, int MODE>
__global__ __launch_bounds__(kWaves * 64, 2) void decode_even_kernel(decode_params p)
{
    static_assert(MODE == 0 || (MODE == 2 && STEP), "plain launches, and score-reuse decode steps of upper layers");
    constexpr int NW = kWaves;
    constexpr int CPR = D / 8, RPI = 64 / CPR, NLD = kTile / RPI, KST = D / 32, XN = 16 / CPR, NPV = 8 / XN;
    constexpr int kUnitD = even_unit_distant(MODE);   // tokens per unit of distant rows
    typedef const __attribute__((address_space(1))) u32x4 *gvec_ptr;
    const decode_hot hot = load_hot_args();
    const int hkv = hot.hkv, prows = hot.prows;
    const int w = blockIdx.x;
    if (w >= p.bal_nwg) {
        if constexpr (STEP) {
            const int pr = w - p.bal_nwg;
            if (pr >= p.npairs) return;
            const int b = pr / hkv, h = pr - b * hkv;
            const int n = load_hlen_arg(b), head_arg = load_head_arg(h);
            if ((MODE == 2 && head_arg < 0) || n < 0) return;
            step_workgroup<D, false, NW, MODE>(p, hot, b, h, n, head_arg);
        }
        return;
    }
    const unsigned long long tr_t0 = p.trace ? wall_clock64() : 0;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int m16 = lane & 15, j = lane >> 4;
    const int kr = lane / CPR, kc = lane % CPR, vc = lane % CPR, vx = (lane / CPR) % XN;
    constexpr int RS = D + 4 * (D / 32) + 1;
    constexpr size_t kTileBytes = sizeof(u32x4) * NW * kTile * CPR, kMergeBytes = sizeof(float) * NW * 16 * RS;
    __shared__ __attribute__((aligned(16))) char lds_raw[kTileBytes > kMergeBytes ? kTileBytes : kMergeBytes];
    __shared__ float sm_m[NW][16], sm_l[NW][16];
    u32x4 *ldsK = (u32x4 *)lds_raw + (size_t)wave * kTile * CPR;
    float *sm_acc = (float *)lds_raw;

    const int g_end = min((w + 1) * p.bal_q, p.bal_total);
    int g = w * p.bal_q;
    // the sequence that holds unit g: the last b with unit_cum[b] * hkv <= g (unit_cum[nseq] * hkv = bal_total > g)
    int b = 0;
    {
        int hi = p.npairs / hkv;
        while (hi - b > 1) { // (at most 8 steps)
            const int mid = (b + hi) >> 1;
            if (load_cum_arg(mid) * hkv <= g) b = mid; else hi = mid;
        }
    }
    const int nseq = p.npairs / hkv;
    while (g < g_end && b < nseq) {
        const int cb = load_cum_arg(b), U = load_cum_arg(b + 1) - cb;   // units per kv head of sequence b
        const int rel = g - cb * hkv;
        if (U <= 0 || rel >= U * hkv) { ++b; continue; }
        const int h = rel / U, u0 = rel - h * U;
        const int cnt = min(U - u0, g_end - g);
        g += cnt;
        const int n = load_hlen_arg(b), head_arg = load_head_arg(h);
        if (MODE == 2 && head_arg < 0) continue; // (a head that starts a block here: not launched so)
        const int n_prox = n < prows ? n : prows, n_dist = n - n_prox;
        const int UD = (n_dist + kUnitD - 1) / kUnitD;
        const size_t pair = (size_t)b * hkv + h;
        const size_t kslot_row = (size_t)(head_arg & 0x7fffffff) + b;

        f32x4 acc[NPV];
#pragma unroll
        for (int x = 0; x < NPV; ++x) acc[x] = f32x4{0.f, 0.f, 0.f, 0.f};
        float m_run = kNegBig, l_run = 0.f;

        // ---- online softmax for head m16 over this lane's 8 tokens (base-2 domain), then O^T += V^T P
        auto softmax_pv = [&](float (&sc)[8], const u32x4 (&vcur)[8]) {
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
#pragma unroll
            for (int x = 0; x < NPV; ++x) {
                u32x4 tlo, thi;
                const int wd = (XN == 1) ? (x >> 1) : x;
                auto dw = [&](const u32x4 &u) -> unsigned { return u[wd]; };
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
        };

        // the part [ua, ub) of a region, in units: its rows [start, end)
        auto rows_of = [&](bool distant, int &start, int &end) {
            const int ua = distant ? u0 : max(u0, UD) - UD, ub = distant ? min(u0 + cnt, UD) : u0 + cnt - UD;
            const int unit = distant ? kUnitD : kUnit;
            start = ua * unit;
            end = min(ub * unit, distant ? n_dist : n_prox);
            return ua < ub && start < end;
        };
        // keys and values of rows [start, end) of one region
        auto walk_kv = [&](const bool distant, const int start, const int end) {
            const int last = end - 1;
            const int excl = (STEP && !distant && n >= prows) ? p.sink + (n - p.sink) % p.window : -1;
            const gvec_ptr Kb = (gvec_ptr)(distant ? hot.kdist + kslot_row * hot.cd * CPR : hot.kprox + pair * prows * CPR);
            const gvec_ptr Vb = (gvec_ptr)(distant ? hot.vdist + pair * hot.cd * CPR : hot.vprox + pair * prows * CPR);
            const pod_bf16 *qsrc = (distant && hot.q_shared && head_arg >= 0) ? hot.q_shared : hot.q;
            u32x4 kreg[NLD], vreg[8];
            int t0 = start + wave * kTile;
            // (from the last tile to the first where a lower layer of the block has just read these keys: see decode_partial_kernel)
            const int ntile_w = t0 < end ? (end - t0 + NW * kTile - 1) / (NW * kTile) : 0;
            const bool rev = p.walk_rev != 0 && distant && head_arg >= 0;
            const int tstep = rev ? -(NW * kTile) : NW * kTile;
            if (rev && ntile_w > 0) t0 += (ntile_w - 1) * (NW * kTile);
#define POD_LOAD_TILE(T0)                                                         \
    _Pragma("unroll") for (int i = 0; i < NLD; ++i) {                             \
        const int row = min((T0) + RPI * i + kr, last);                           \
        kreg[i] = Kb[(size_t)row * CPR + kc];                                     \
    }                                                                             \
    _Pragma("unroll") for (int e = 0; e < 8; ++e) {                               \
        const int tok = (e < 4) ? 4 * j + e : 16 + 4 * j + (e - 4);               \
        const int row = min((T0) + tok, last);                                    \
        vreg[e] = __builtin_nontemporal_load(&Vb[(size_t)row * CPR + vc]);        \
    }
            if (ntile_w > 0) { POD_LOAD_TILE(t0) }
            bf16x8 qf[KST];
            {
                const gvec_ptr qrow = (gvec_ptr)(qsrc + ((size_t)b * hot.hq + (size_t)h * hot.rep + m16) * D);
#pragma unroll
                for (int s = 0; s < KST; ++s) {
                    u32x4 t = u32x4{0u, 0u, 0u, 0u};
                    if (m16 < hot.rep) t = qrow[4 * s + j];
                    qf[s] = as_bf16x8(t);
                }
            }
            for (int it = 0; it < ntile_w; ++it, t0 += tstep) {
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
                // the next tile's loads go out as soon as the registers are free (K is in LDS, V is copied)
                if (it + 1 < ntile_w) { POD_LOAD_TILE(t0 + tstep) }
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
                float sc[8];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int tok0 = t0 + 4 * j + i, tok1 = tok0 + 16;
                    sc[i] = (tok0 < end && (!STEP || tok0 != excl)) ? s0[i] * hot.scale_log2e : kNegBig;
                    sc[4 + i] = (tok1 < end && (!STEP || tok1 != excl)) ? s1[i] * hot.scale_log2e : kNegBig;
                }
                softmax_pv(sc, vcur);
            }
#undef POD_LOAD_TILE
        };
        // Score reuse, upper layer, distant rows [start, end): their logits are the lowest layer's, stored tile by tile in
        // the per-lane order of the S^T accumulators; only V is streamed, two tiles in flight per wave.
        auto walk_sv = [&](const int start, const int end) {
            const int last = end - 1;
            const gvec_ptr Vb = (gvec_ptr)(hot.vdist + pair * hot.cd * CPR);
            u32x4 vreg[8];
            int t0 = start + wave * kTile;
                typedef const __attribute__((address_space(1))) f32x4 *gf4_r;
                const gf4_r sbase = (gf4_r)(p.scores + pair * p.score_stride * hot.rep) + ((size_t)j * hot.rep + (m16 < hot.rep ? m16 : 0)) * 2;
                f32x4 sregA[2], sregB[2];
                u32x4 vregB[8];
#define POD_LOAD_SV(SR, VR, T0)                                                   \
                {                                                                     \
                    const gf4_r sp = sbase + (size_t)(min((T0), last) >> 5) * 8 * hot.rep; \
                    SR[0] = sp[0];                                                    \
                    SR[1] = sp[1];                                                    \
                }                                                                     \
                _Pragma("unroll") for (int e = 0; e < 8; ++e) {                       \
                    const int tok = (e < 4) ? 4 * j + e : 16 + 4 * j + (e - 4);       \
                    const int row = min((T0) + tok, last);                            \
                    VR[e] = __builtin_nontemporal_load(&Vb[(size_t)row * CPR + vc]);  \
                }
#define POD_CONSUME_SV(SR, VR, T0, TNEXT)                                         \
                {                                                                     \
                    u32x4 vcur[8];                                                    \
                    float sc[8];                                                      \
                    _Pragma("unroll") for (int e = 0; e < 8; ++e) vcur[e] = VR[e];    \
                    _Pragma("unroll") for (int i = 0; i < 4; ++i) {                   \
                        const int tok0 = (T0) + 4 * j + i, tok1 = tok0 + 16;          \
                        sc[i] = tok0 < end ? SR[0][i] : kNegBig;                      \
                        sc[4 + i] = tok1 < end ? SR[1][i] : kNegBig;                  \
                    }                                                                 \
                    if (m16 >= hot.rep) {                                             \
                        _Pragma("unroll") for (int i = 0; i < 8; ++i) sc[i] = 0.f; /* padding heads: any finite value */ \
                    }                                                                 \
                    if ((TNEXT) < end) { POD_LOAD_SV(SR, VR, TNEXT) }                 \
                    softmax_pv(sc, vcur);                                             \
                }
                constexpr int kStep = NW * kTile;
                if (t0 < end) { POD_LOAD_SV(sregA, vreg, t0) }
                if (t0 + kStep < end) { POD_LOAD_SV(sregB, vregB, t0 + kStep) }
                for (; t0 < end; t0 += 2 * kStep) {
                    POD_CONSUME_SV(sregA, vreg, t0, t0 + 2 * kStep)
                    if (t0 + kStep < end) POD_CONSUME_SV(sregB, vregB, t0 + kStep, t0 + 3 * kStep)
                }
#undef POD_CONSUME_SV
#undef POD_LOAD_SV
        };
        {
            int start, end;
            if constexpr (MODE == 2) {
                if (rows_of(true, start, end)) walk_sv(start, end);
                if (rows_of(false, start, end)) walk_kv(false, start, end);
            } else {
                for (int part = 0; part < 2; ++part)
                    if (rows_of(part == 0, start, end)) walk_kv(part == 0, start, end);
            }
        }

        // ---- this workgroup's partial of the pair: merge the waves, store it in the pair's slot w - w_lo
        __syncthreads(); // all waves are done with their K tiles
        if (m16 < hot.rep) {
#pragma unroll
            for (int x = 0; x < NPV; ++x)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int slot = 4 * j + i;
                    const int dim = (XN == 1) ? 8 * slot + x : 8 * (slot % 8) + 2 * x + slot / 8;
                    sm_acc[((size_t)wave * hot.rep + m16) * RS + dim + 4 * (dim >> 5)] = acc[x][i];
                }
            if (j == 0) { sm_m[wave][m16] = m_run; sm_l[wave][m16] = l_run; }
        }
        __syncthreads();
        const int NC = hot.nc + (STEP ? 1 : 0);
        const int w_lo = (cb * hkv + h * U) / p.bal_q;
        for (int t = threadIdx.x; t < hot.rep * D; t += blockDim.x) {
            const int head = t / D, dim = t % D;
            float M = sm_m[0][head];
#pragma unroll
            for (int v = 1; v < NW; ++v) M = fmaxf(M, sm_m[v][head]);
            float A = 0.f, Lsum = 0.f;
#pragma unroll
            for (int v = 0; v < NW; ++v) {
                const float f = exp2f(sm_m[v][head] - M);
                A += f * sm_acc[((size_t)v * hot.rep + head) * RS + dim + 4 * (dim >> 5)];
                Lsum += f * sm_l[v][head];
            }
            typedef __attribute__((address_space(1))) float *gfloat_ptr;
            const size_t slot = ((size_t)b * hot.hq + (size_t)h * hot.rep + head) * NC + (w - w_lo);
            ((gfloat_ptr)hot.part_acc)[slot * D + dim] = A;
            if (dim == 0) { ((gfloat_ptr)hot.part_ml)[slot * 2] = M; ((gfloat_ptr)hot.part_ml)[slot * 2 + 1] = Lsum; }
        }
        __syncthreads(); // the merge buffer is the next pair's K tiles
    }
    if (p.trace && threadIdx.x == 0 && w < p.trace_cap) { // measurement aid: workgroup, XCD and CU, clock at start and end
        unsigned long long *t = p.trace + 8 * (size_t)w;
        t[0] = (unsigned long long)w;
        t[1] = (unsigned long long)xcc_id() | ((unsigned long long)__builtin_amdgcn_s_getreg((32 - 1) << 11 | 4) << 8);
        t[2] = tr_t0; t[3] = tr_t0; t[6] = wall_clock64();
    }
}

// One workgroup per (query head, sequence): merge the chunk partials, normalise, round to bf16.
// Merging two partials brought to a common max is the paper's gate (Eq. 4) applied to unnormalised
// sums; over many chunks it is the same running-max merge the partial kernel uses over tiles.
// Like the partial kernel it starts from the host mirror's length so that its loads of the
// partials go out together with the loads that validate that length; the validation only gates
// the final store.
template <int D, int kCombineThreads = 256, int UN = 8, int DS = D>
__global__ __launch_bounds__(kCombineThreads) void decode_combine_kernel(decode_params p)
{
    // DS = dims per workgroup: blockIdx.z picks a slice of the head dimension, so that a head's
    // partials are pulled through several CUs; every slice recomputes the same chunk weights
    constexpr int LPR = DS / 4;      // lanes per partial row slice (float4 each)
    constexpr int ROW = D / 4;       // float4 per partial row
    const int xs = blockIdx.z * LPR;
    constexpr int NG = kCombineThreads / LPR; // chunk groups
    typedef const __attribute__((address_space(1))) float *gfloat_ptr;
    typedef const __attribute__((address_space(1))) f32x4 *gf4_ptr;
    typedef const __attribute__((address_space(1))) int32_t *gint_ptr;
    const int head = blockIdx.x, b = blockIdx.y;
    const decode_hot hot = load_hot_args();
    const int n_host = load_hlen_arg(b);
    const bool step = p.step != 0;   // the partials of a decode step: the pieces of the rows held before the new token
                                     // plus the step's own partial in slot hot.nc, whose normaliser says whether the step was valid
    bool bad = false;
    int n = n_host;
    if (!hot.use_hlen) {
        if (step) {
            n = p.positions[b];
            if (n < 0 || n >= p.maxctx || n >= p.max_len) { bad = true; n = -1; }
        } else {
            n = decode_seq_len(p, b, &bad);
        }
    }
    // validation inputs (independent loads, consumed at the very end)
    int v_ctx = 0, v_dev = 0, v_low = 0;
    if (!step) { v_ctx = ((gint_ptr)hot.ctx)[b]; v_dev = ((gint_ptr)hot.lens_layer)[b]; v_low = ((gint_ptr)hot.lens_lowest)[b]; }

    const int nn = n > 0 ? n : 0;
    const int n_prox = nn < hot.prows ? nn : hot.prows;
    const int n_dist = nn - n_prox;
    const int chunk_d = hot.chunk & 0xffff, chunk_p = (int)((unsigned)hot.chunk >> 16);
    int nd = min((n_dist + chunk_d - 1) / chunk_d, hot.max_nd);
    int np = min((n_prox + chunk_p - 1) / chunk_p, hot.nc - hot.max_nd);
    if (p.bal_q > 0) { // even split: the pair's partials are those of the workgroups its units fall to, in its first slots
        const int U = (n_dist + p.bal_unit_d - 1) / p.bal_unit_d + (n_prox + kUnit - 1) / kUnit;
        const int g0 = load_cum_arg(b) * hot.hkv + (head / hot.rep) * U;
        nd = U > 0 ? (g0 + U - 1) / p.bal_q - g0 / p.bal_q + 1 : 0;
        np = 0;
    }
    const int NC = hot.nc + (step ? 1 : 0);
    const int nvalid = step ? (n >= 0 ? nd + np + 1 : 0) : (n > 0 ? nd + np : 0);
    const gfloat_ptr ml = (gfloat_ptr)hot.part_ml + ((size_t)b * hot.hq + head) * NC * 2;
    const gf4_ptr pa = (gf4_ptr)hot.part_acc + ((size_t)b * hot.hq + head) * NC * ROW + xs;
    auto chunk_slot = [&](int v) { return v < nd ? v : (v < nd + np ? hot.max_nd + (v - nd) : hot.nc); };
    if (step && n >= 0 && ml[hot.nc * 2 + 1] < 0.f) { bad = true; n = -1; }   // the step's own validation failed

    const int g = threadIdx.x / LPR, x = threadIdx.x % LPR;
    const int head_arg = load_head_arg(head / hot.rep);
    const bool low = head_arg < 0;   // this layer is the lowest of the head's block
    // gated upper layer: a head whose gate reached tau merges its proximal partials only
    int v_begin = 0;
    if (p.mode == 3 && !low && nd > 0 && p.skip[(size_t)b * hot.hq + head] != 0) v_begin = nd;
    // lowest layer of a score-reuse block: leave the distant maximum and sum for the gates of the upper layers
    if (p.mode != 0 && low && !step && xs == 0 && threadIdx.x < 64) {
        const float2 dl = merged_ml((const float *)ml, n > 0 ? nd : 0, (int)threadIdx.x);
        if (threadIdx.x == 0) {
            p.gate_d[((size_t)b * hot.hq + head) * 2] = dl.x;
            p.gate_d[((size_t)b * hot.hq + head) * 2 + 1] = dl.y;
            if (head % hot.rep == 0) p.score_hdr[4 * ((size_t)b * hot.hkv + head / hot.rep) + 3] = 1;
        }
    }
    float m_run = kNegBig, l_run = 0.f;
    f32x4 a = {0.f, 0.f, 0.f, 0.f};
    for (int v0 = v_begin + g; v0 < nvalid; v0 += NG * UN) {
        float mk[UN], lk[UN];
        f32x4 ak[UN];
#pragma unroll
        for (int k = 0; k < UN; ++k) {
            const int v = v0 + k * NG;
            const int cs = chunk_slot(v < nvalid ? v : v0);
            mk[k] = ml[cs * 2];
            lk[k] = ml[cs * 2 + 1];
            ak[k] = pa[(size_t)cs * ROW + x];
            if (v >= nvalid) { mk[k] = kNegBig; lk[k] = 0.f; ak[k] = f32x4{0.f, 0.f, 0.f, 0.f}; }
        }
        float mb = mk[0];
#pragma unroll
        for (int k = 1; k < UN; ++k) mb = fmaxf(mb, mk[k]);
        const float m_new = fmaxf(m_run, mb);
        const float alpha = exp2f(m_run - m_new);
        a *= alpha;
        l_run *= alpha;
#pragma unroll
        for (int k = 0; k < UN; ++k) {
            const float f = exp2f(mk[k] - m_new);
            a += f * ak[k];
            l_run += f * lk[k];
        }
        m_run = m_new;
    }
    __shared__ f32x4 sa[NG][LPR];
    __shared__ float sm[NG], sl[NG];
    sa[g][x] = a;
    if (x == 0) { sm[g] = m_run; sl[g] = l_run; }
    __syncthreads();
    if (g != 0) return;
    float M = sm[0];
#pragma unroll
    for (int k = 1; k < NG; ++k) M = fmaxf(M, sm[k]);
    f32x4 o = {0.f, 0.f, 0.f, 0.f};
    float L = 0.f;
#pragma unroll
    for (int k = 0; k < NG; ++k) {
        const float f = exp2f(sm[k] - M);
        o += f * sa[k][x];
        L += f * sl[k];
    }
    // validation: the same rule as decode_seq_len, on the values loaded at the top
    if (hot.use_hlen && !step) {
        if (v_ctx == 0) n = 0;
        else if (v_ctx < 0 || v_ctx > p.maxctx || v_ctx > p.max_len || v_ctx != v_dev || (v_ctx > hot.prows && v_low != v_ctx) || v_ctx != n_host) {
            bad = true;
            n = 0;
        }
    }
    const int n_ctx = step && n >= 0 ? n + 1 : n;   // the context the attention is over
    if (p.mode != 0 && !low && n_ctx > hot.prows) { // the distant logits must be those of this token and of the head's block
        const size_t tag = 4 * ((size_t)b * hot.hkv + head / hot.rep);
        if (p.score_hdr[tag] != n_ctx || p.score_hdr[tag + 1] != (head_arg & 0x7fffffff) ||
            p.score_hdr[tag + 2] != __float_as_int(hot.scale_log2e) || (p.mode == 3 && p.score_hdr[tag + 3] != 1)) { bad = true; n = step ? -1 : 0; }
    }
    uint2 res = make_uint2(0u, 0u);
    if (step ? n >= 0 : n > 0) {
        const float inv = 1.f / L;
        res.x = pack_bf16(o.x * inv, o.y * inv);
        res.y = pack_bf16(o.z * inv, o.w * inv);
    } else if (bad && head == 0 && x == 0 && xs == 0) {
        atomicOr(p.flag, 2);
    }
    ((uint2 *)(p.out + ((size_t)b * hot.hq + head) * D))[xs + x] = res;
}

int chunk_slots(int rows, int chunk) { return (rows + chunk - 1) / chunk; }

} // namespace

// ---------------------------------------------------------------------------------------------
// Split-K partials in library-owned memory, for callers that may not allocate (code under HIP
// graph capture, serving loops, harnesses that forbid hipMalloc): a fixed array in the code
// object's device data, one copy per GPU, held until the process ends.  In host code the array's
// name is only a stand-in for the symbol; its device address is looked up once per device and
// that pointer is what kernels, copies and clears receive.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];       // device address of `scratch` on device i (NULL: not looked up yet)
std::mutex g_scratch_mutex;
} // namespace

// Measurement aid: the plainest kernel that reads `bytes` once: one resident round of workgroups (2 per CU), each
// walking its own contiguous part with 8 x 16 bytes in flight per thread, results folded into a word nobody stores.
// Non-temporal loads: the fastest plain read found on this chip (134 MB cold: 21.4-22.4 us against 24.7 us with
// ordinary loads; 1-2 GB: 7.0-7.2 against 6.1-6.4 TB/s).  What it reaches on cold memory is the ceiling a streaming
// launch of that size can be held to on this device.
__device__ unsigned pod_stream_read_sink; // (external linkage: a store the compiler cannot prove dead)
namespace {
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4 *__restrict__ src, size_t n16, size_t per_wg)
{
    typedef const __attribute__((address_space(1))) u32x4 *gvec_ptr;
    const size_t lo = (size_t)blockIdx.x * per_wg, hi = lo + per_wg < n16 ? lo + per_wg : n16;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (size_t i = lo + threadIdx.x; i < hi; i += 8 * 256) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = i + (size_t)u * 256 < hi ? __builtin_nontemporal_load(&((gvec_ptr)src)[i + (size_t)u * 256]) : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
    }
    if ((acc.x ^ acc.y) == 0x9e3779b9u && (acc.z ^ acc.w) == 0x7f4a7c15u) pod_stream_read_sink = acc.x; // practically never
}
} // namespace

int pod_launch_stream_read(pod_cache *c, const void *buf, size_t bytes, hipStream_t st)
{
    const size_t n16 = bytes / 16;
    int dev = 0, cus = 256;
    POD_HIP_TRY(hipGetDevice(&dev));
    POD_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    size_t grid = (size_t)2 * cus;
    size_t per_wg = (n16 + grid - 1) / grid;
    per_wg = (per_wg + 255) / 256 * 256;
    grid = (n16 + per_wg - 1) / per_wg;
    const bool prof = c && c->prof_ev && c->prof_n < c->prof_cap;   // timed like the decode kernel's launches
    if (prof) POD_HIP_TRY(hipEventRecord(c->prof_ev[2 * c->prof_n], st));
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)grid), dim3(256), 0, st, (const u32x4 *)buf, n16, per_wg);
    if (prof) { POD_HIP_TRY(hipEventRecord(c->prof_ev[2 * c->prof_n + 1], st)); c->prof_n += 1; }
    POD_HIP_TRY(hipGetLastError());
    return POD_OK;
}

namespace {
__global__ void xcc_probe_kernel(int32_t *out) { if (threadIdx.x == 0) out[blockIdx.x] = xcc_id(); }
struct xcd_map { bool probed; int nxcd; };
xcd_map g_xcd[kMaxDevices];
} // namespace

// Over how many XCDs does a one-dimensional launch spread its workgroups round-robin?  Probed once per device with a
// launch of 256 workgroups that record their XCC_ID: k = number of distinct ids, accepted if workgroup w reports the
// same id as workgroup w mod k and the first k ids are all different.  *nxcd = k, or 0 (no such pattern: the
// XCD-local hand-off is not used).  Which XCD a position lands on may differ from launch to launch; only the modulus
// is taken from here, and every launch checks its own placement.
int pod_probe_xcds(int *nxcd)
{
    int dev = -1;
    POD_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return pod_fail(POD_ERR_INVALID_ARG, "device %d outside [0, %d)", dev, kMaxDevices);
    void *buf = nullptr;
    size_t bytes = 0;
    int rc = pod_decode_static_scratch(&buf, &bytes);
    if (rc) return rc;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    xcd_map &m = g_xcd[dev];
    if (!m.probed) {
        constexpr int kProbe = 256;
        int32_t ids[kProbe];
        hipLaunchKernelGGL(xcc_probe_kernel, dim3(kProbe), dim3(64), 0, 0, (int32_t *)buf);
        POD_HIP_TRY(hipGetLastError());
        POD_HIP_TRY(hipMemcpy(ids, buf, sizeof ids, hipMemcpyDeviceToHost));   // (waits for the probe)
        int k = 0;
        bool seen[16] = {};
        for (int w = 0; w < kProbe; ++w)
            if (ids[w] >= 0 && ids[w] < 16 && !seen[ids[w]]) { seen[ids[w]] = true; ++k; }
        bool ok = k >= 1 && k <= 16;
        for (int w = 0; ok && w < kProbe; ++w) ok = ids[w] >= 0 && ids[w] < 16 && ids[w] == ids[w % k];
        for (int x = 0; ok && x < k; ++x)
            for (int y = 0; y < x; ++y) ok = ok && ids[x] != ids[y];
        m.nxcd = ok ? k : 0;
        m.probed = true;
    }
    *nxcd = m.nxcd;
    return POD_OK;
}

int pod_decode_static_scratch(void **ptr, size_t *bytes)
{
    int dev = -1;
    POD_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return pod_fail(POD_ERR_INVALID_ARG, "device %d outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        POD_HIP_TRY(hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch)));   // of the current device's copy
        if (!p) return pod_fail(POD_ERR_HIP, "hipGetSymbolAddress returned a NULL address");
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    *bytes = kStaticScratchBytes;
    return POD_OK;
}

size_t pod_decode_workspace_bytes(const pod_layout &ly)
{
    const size_t nc = (size_t)chunk_slots(ly.Cd, kMinChunk) + chunk_slots(ly.P, kMinChunk) + 2;
    const size_t bytes = (size_t)ly.B * ly.Hq * nc * (ly.D + 2) * sizeof(float);
    return (bytes + 255) / 256 * 256;
}

size_t pod_score_stride(const pod_layout &ly) { return ((size_t)ly.Cd + kTile - 1) / kTile * kTile; } // whole tiles

// header of the score buffer: int32 [B][Hkv][4] tags, float [B][Hq][2] distant (max, sum), int32 [B][Hq] skip flags
static size_t score_tag_bytes(const pod_layout &ly) { return ((size_t)ly.B * ly.Hkv * 4 * sizeof(int32_t) + 255) / 256 * 256; }
static size_t score_gate_bytes(const pod_layout &ly) { return ((size_t)ly.B * ly.Hq * 2 * sizeof(float) + 255) / 256 * 256; }
static size_t score_skip_bytes(const pod_layout &ly) { return ((size_t)ly.B * ly.Hq * sizeof(int32_t) + 255) / 256 * 256; }
size_t pod_score_skip_offset_bytes(const pod_layout &ly) { return score_tag_bytes(ly) + score_gate_bytes(ly); }
size_t pod_score_header_bytes(const pod_layout &ly) { return score_tag_bytes(ly) + score_gate_bytes(ly) + score_skip_bytes(ly); }

// The split-K plan of a decode launch: host logic only, a function of the shape (also exported for the CPU tests).
// Chunk size, for workgroups of nw waves (8 / nw of them fit a CU).  Small problems (config 2: 262K rows) want
// exactly one resident round of workgroups: rows / (CUs x 8 / nw).  Large or ragged problems want many rounds
// of moderately sized chunks so that the tail stays short: measured best near 256 tokens per wave for
// 16 ragged sequences of 4K-32K tokens and within 2 % of best for 4 sequences of 128K.
// Never below one tile per wave, so the partials stay a small fraction of the K/V bytes.
// env_chunk, env_chunk_prox: tuning / test overrides (0 = none); scores: a score-reuse or gated call; small_prox: the
// gated form's proximal launch.
// reader: a score-reuse step of an upper layer in one launch: its distant pieces stream values and logits but no keys,
// about half the bytes per token of a proximal piece, so they take about twice the tokens.
pod_decode_plan_t pod_plan_decode(int cus, int B, int Hkv, int P, int max_len, int env_chunk, int env_chunk_prox, bool scores,
                                  bool small_prox, bool fused_allowed, bool reader)
{
    const int npairs = B * Hkv;
    const long rows = (long)max_len * npairs;
    const int max_prox = max_len < P ? max_len : P;
    const int max_dist = max_len - max_prox;
    auto plan = [&](int nw) {
        const long min_chunk = (long)kTile * nw, auto_max = 256L * nw, round = (long)cus * 8 / nw;
        long chunk = env_chunk > 0 ? env_chunk : rows / round;
        chunk = (chunk + kTile - 1) / kTile * kTile;
        if (chunk < min_chunk) chunk = min_chunk;
        if (chunk > auto_max && env_chunk <= 0) chunk = auto_max;
        if (chunk > 8192) chunk = 8192;
        // Proximal chunks.  In the gated form the proximal region is a launch of its own, whose duration is the time
        // of one workgroup: its waves walk their tiles one after the other.  There the region is cut into the smallest
        // chunks (one tile per wave); everywhere else proximal and distant workgroups take equally many tokens.
        long chunk_p = env_chunk_prox > 0 ? env_chunk_prox : (small_prox ? min_chunk : chunk);
        chunk_p = (chunk_p + kTile - 1) / kTile * kTile;
        if (chunk_p < min_chunk) chunk_p = min_chunk;
        if (chunk_p > 8192) chunk_p = 8192;
        // Where the rule above lands just past one resident round (the proximal region's ragged last piece, a distant
        // region a few tokens over a multiple of the chunk), the workgroups beyond it start only when a first one
        // has left, near the end of the launch, and the launch ends that much later (measured on the 32K-token shape:
        // 8 of 520 workgroups started at 18 us of a 30 us launch).  There the distant pieces keep their size (or grow
        // tile by tile) and the proximal region is cut into the slots that are left.
        const long resident = round / npairs;
        if (env_chunk <= 0 && env_chunk_prox <= 0 && !scores && resident >= 2 && chunk <= auto_max &&
            chunk_slots(max_dist, (int)chunk) + chunk_slots(max_prox, (int)chunk_p) > resident)
            for (long t = chunk; t <= auto_max + 8 * kTile; t += kTile) {
                const long left = resident - chunk_slots(max_dist, (int)t);
                if (left < 1) continue;
                long tp = ((max_prox + left - 1) / left + kTile - 1) / kTile * kTile;
                if (tp < min_chunk) tp = min_chunk;
                if (tp > 2 * t) continue;
                chunk = t;
                chunk_p = tp;
                break;
            }
        if (reader && env_chunk <= 0 && env_chunk_prox <= 0 && resident >= 2) {
            // one resident round whose longest piece (in bytes) is as short as possible: a distant token counts 17 / 32
            // of a proximal one (values + 4 bytes of logit per query head against keys + values)
            long best = -1, best_t = chunk, best_tp = chunk_p;
            for (long t = min_chunk; t <= 4096; t += kTile) {
                const long left = resident - chunk_slots(max_dist, (int)t);
                if (left < 1) continue;
                long tp = ((max_prox + left - 1) / left + kTile - 1) / kTile * kTile;
                if (tp < min_chunk) tp = min_chunk;
                if (tp > 8192) continue;
                const long cost = t * 17 > tp * 32 ? t * 17 : tp * 32;
                if (best < 0 || cost < best) { best = cost; best_t = t; best_tp = tp; }
            }
            if (best >= 0) { chunk = best_t; chunk_p = best_tp; }
        }
        pod_decode_plan_t r;
        r.waves = nw;
        r.chunk = (int)chunk; r.chunk_p = (int)chunk_p;
        r.max_nd = chunk_slots(max_dist, (int)chunk);
        r.nc = r.max_nd + chunk_slots(max_prox, (int)chunk_p);
        r.merge_inside = false;
        return r;
    };
    // Merge inside the streaming kernel only where the launch is about one resident round of workgroups:
    // a workgroup waits for its arrival to be counted before it leaves, and in a launch of several rounds that wait
    // keeps the next workgroup from starting (measured: 4 sequences of 128K tokens 13.1 ms per step against 12.0 ms
    // with the separate merge kernel).  Such launches run workgroups of 8 waves, all others of kWaves.
    pod_decode_plan_t pl = plan(fuse_waves(1));
    pl.merge_inside = !scores && fused_allowed && (long)pl.nc * npairs <= (long)cus * 5 / 4;
    if (!pl.merge_inside) pl = plan(kWaves);
    return pl;
}

// The even split of a plain launch (host logic): lens[b] tokens per sequence (<= 0: none), `slots` workgroups at most.
// unit_cum[b] = units (unit_d tokens of distant rows, then kUnit tokens of proximal rows, each region's last unit may
// be short) of the sequences before b, per kv head.  All units stand in one line, sequence after sequence, kv head after kv head
// inside a sequence; workgroup w takes units [w q, (w + 1) q).  most = partials of the pair cut into most parts.
// Returns false if there is nothing to split.
bool pod_plan_even(int slots, int B, int Hkv, int P, int unit_d, const int32_t *lens, int32_t *unit_cum, pod_even_plan_t *pl)
{
    unit_cum[0] = 0;
    for (int b = 0; b < B; ++b) {
        const int n = lens[b] > 0 ? lens[b] : 0, n_prox = n < P ? n : P;
        unit_cum[b + 1] = unit_cum[b] + (n - n_prox + unit_d - 1) / unit_d + (n_prox + kUnit - 1) / kUnit;
    }
    const long total = (long)unit_cum[B] * Hkv;
    if (total <= 0 || total > 0x3fffffff || slots < 1) return false;
    const long q = (total + slots - 1) / slots;
    pl->q = (int32_t)q; pl->total = (int32_t)total; pl->nwg = (int32_t)((total + q - 1) / q);
    int most = 1;
    for (int b = 0; b < B; ++b) {
        const long U = unit_cum[b + 1] - unit_cum[b];
        for (int h = 0; h < Hkv && U > 0; ++h) {
            const long g0 = (long)unit_cum[b] * Hkv + h * U;
            const int parts = (int)((g0 + U - 1) / q - g0 / q) + 1;
            most = parts > most ? parts : most;
        }
    }
    pl->most = most;
    return true;
}

int pod_launch_decode(const pod_cache *c, int layer, const void *q, const void *q_shared, const int32_t *ctx, int B,
                      int max_len, float scale, void *ws, size_t ws_bytes, void *scores, float tau, void *out,
                      hipStream_t st, const pod_step_args *step)
{
    const pod_layout &ly = c->ly;
    const size_t row16 = (size_t)ly.D / 8; // u32x4 per row
    const int H = ly.Hkv;
    bool lowest_all = true, lowest_any = false;
    for (int h = 0; h < H; ++h) {
        const bool low = c->lowest[(size_t)layer * H + h] == layer;
        lowest_all = lowest_all && low;
        lowest_any = lowest_any || low;
    }
    // the layer whose lengths the device compares with this layer's: the block's lowest layer when all kv heads
    // share it (the host has already compared every head's lowest layer through its mirror)
    const int lowest = c->uniform ? c->lowest[(size_t)layer * H] : layer;
    decode_params p;
    const pod_headmap hm = pod_make_headmap(c, layer);
    for (int h = 0; h < H; ++h) p.head_arg[h] = hm.kslot_row[h] | (((hm.lowest_mask >> h) & 1) ? (int32_t)0x80000000 : 0);
    p.hot.kdist = (const u32x4 *)(c->base + ly.off_distK);
    p.hot.vdist = (const u32x4 *)(c->base + ly.off_distV) + pod_dist_row0(ly, layer, 0, 0) * row16;
    p.hot.kprox = (const u32x4 *)(c->base + ly.off_proxK) + pod_prox_row0(ly, layer, 0, 0) * row16;
    p.hot.vprox = (const u32x4 *)(c->base + ly.off_proxV) + pod_prox_row0(ly, layer, 0, 0) * row16;
    p.hot.cd = ly.Cd; p.hot.prows = ly.P; p.hot.hkv = ly.Hkv; p.hot.rep = ly.rep; p.hot.hq = ly.Hq;
    p.hot.q = (const pod_bf16 *)q; p.hot.q_shared = (const pod_bf16 *)q_shared;
    p.hot.scale_log2e = scale * 1.4426950408889634f;
    p.hot.ctx = ctx;
    p.hot.lens_layer = (const int32_t *)(c->base + ly.off_lens) + (size_t)layer * ly.B;
    p.hot.lens_lowest = (const int32_t *)(c->base + ly.off_lens) + (size_t)lowest * ly.B;
    p.flag = (int32_t *)(c->base + ly.off_flag);
    p.maxctx = ly.maxctx;
    p.max_len = max_len;
    p.out = (pod_bf16 *)out;
    p.mode = scores ? (tau >= 0.f ? 3 : 2) : 0;
    p.score_hdr = (int32_t *)scores;
    p.gate_d = scores ? (float *)((char *)scores + score_tag_bytes(ly)) : nullptr;
    p.skip = scores ? (int32_t *)((char *)scores + score_tag_bytes(ly) + score_gate_bytes(ly)) : nullptr;
    p.tau = tau;
    p.scores = scores ? (float *)((char *)scores + pod_score_header_bytes(ly)) : nullptr;
    p.score_stride = (int32_t)pod_score_stride(ly);
    p.tickets = (unsigned long long *)(c->base + ly.off_tickets);
    p.step_done = (int32_t *)(c->base + ly.off_stepdone);
    p.k_new = step ? (const u32x4 *)step->k_new : nullptr;
    p.v_new = step ? (const u32x4 *)step->v_new : nullptr;
    p.positions = step ? step->positions : nullptr;
    p.lens_w = (int32_t *)(c->base + ly.off_lens) + (size_t)layer * ly.B;
    p.low_is_self = lowest == layer;
    p.sink = ly.S; p.window = ly.W;
    p.trace = (unsigned long long *)c->trace; p.trace_cap = c->trace_cap;
    // layers of a block take turns in the direction they walk the block's distant keys (the lowest layer forward)
    p.walk_rev = c->walk_turns ? ((layer - c->lowest[(size_t)layer * H]) & 1) : 0;
    // 0: separate combine kernel; 1: the last workgroup of a (sequence, kv head) pair merges; 2: 1 + the cache update
    p.step = step ? 1 : 0;
    // XCD-local hand-off: only where the pairs spread evenly over the XCDs (else some XCDs would sit idle)
    const int npairs = B * ly.Hkv;
    p.nxcd = c->nxcd > 0 ? c->nxcd : 1;
    p.npairs = npairs;
    p.hot.use_hlen = B <= kMaxHostLens && !c->device_lengths;
    if (p.hot.use_hlen)
        for (int b = 0; b < B; ++b) p.hlen[b] = (int32_t)c->host_len[(size_t)layer * ly.B + b];

    int cus = 256;
    (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device);
    // A score-reuse step: the step forms of the writing launch (kv heads whose block starts at this layer) and of
    // the reading launch (the others); a layer with heads of both kinds takes both.  (No gated form.)
    const bool reuse_step = step && scores;
    if (reuse_step && tau >= 0.f) return pod_fail(POD_ERR_INVALID_ARG, "a decode step has no gated form");
    const pod_decode_plan_t pl = pod_plan_decode(cus, B, ly.Hkv, ly.P, max_len, c->tune_chunk, c->tune_chunk_prox, scores && !reuse_step,
                                                 scores && !lowest_all && tau >= 0.f, c->fused_merge != 0, reuse_step && !lowest_any);
    const bool merge_inside = pl.merge_inside;
    p.hot.chunk = (int)((unsigned)pl.chunk | ((unsigned)pl.chunk_p << 16));
    p.hot.max_nd = pl.max_nd;
    p.hot.nc = pl.nc;
    // The even split (decode_even_kernel) for plain launches of several rounds whose lengths the host knows: one round
    // of two workgroups per CU, every workgroup the same number of kUnit-token units.
    p.bal_q = 0; p.bal_nwg = 0; p.bal_total = 0;
    // (score reuse: the decode step of a layer none of whose kv heads starts a block.  A layer that writes the logits
    // gains nothing from it: 16 sequences 218 us either way, 4 x 128K tokens 399 against 387 us.)
    const int even_mode = reuse_step ? 2 : 0;
    bool even = !merge_inside && p.hot.use_hlen && c->even_split && (p.mode == 0 || (reuse_step && !lowest_any));
    p.bal_unit_d = even_unit_distant(even_mode);
    if (even) {
        pod_even_plan_t ev;
        even = pod_plan_even(2 * cus, B, H, ly.P, p.bal_unit_d, p.hlen, p.unit_cum, &ev);
        // (a batch of one very long and many short sequences cuts the long one into more parts than fixed pieces
        // would: where the caller's scratch does not hold them the launch keeps to fixed pieces)
        if (even && (size_t)B * ly.Hq * ((size_t)ev.most + (step ? 1 : 0)) * (ly.D + 2) * sizeof(float) > ws_bytes) even = false;
        if (even) {
            p.bal_q = ev.q; p.bal_total = ev.total; p.bal_nwg = ev.nwg;
            p.hot.nc = ev.most; p.hot.max_nd = ev.most;
        }
    }
    const size_t NC = (size_t)p.hot.nc + (step ? 1 : 0); // partial slots per query head (a step keeps one more)
    const size_t acc_bytes = (size_t)B * ly.Hq * NC * ly.D * sizeof(float);
    const size_t ml_bytes = (size_t)B * ly.Hq * NC * 2 * sizeof(float);
    if (acc_bytes + ml_bytes > ws_bytes)
        return pod_fail(POD_ERR_CAPACITY, "decode scratch too small: %d sequences x %d query heads x %zu chunks of up to %d tokens need %zu bytes, %zu are there",
                        B, ly.Hq, NC, max_len, acc_bytes + ml_bytes, ws_bytes);
    p.hot.part_acc = (float *)ws;
    p.hot.part_ml = (float *)((char *)ws + acc_bytes);

    const size_t WGS = (size_t)p.hot.nc;   // workgroups per (sequence, kv head) pair
    p.slots = (int32_t)WGS;
    const int fuse = step ? (merge_inside ? 2 : 3) : (merge_inside ? 1 : 0);
    const bool loc = merge_inside && c->xcd_local && c->nxcd >= 1 && (npairs % c->nxcd == 0 || npairs >= 8 * c->nxcd);
    const size_t loc_wgs = (size_t)((npairs + p.nxcd - 1) / p.nxcd) * p.nxcd * WGS;
    if (loc && loc_wgs > 0x7fffffffu) return pod_fail(POD_ERR_CAPACITY, "launch too large");
    const dim3 grid = loc ? dim3((unsigned)loc_wgs) : dim3((unsigned)WGS, (unsigned)ly.Hkv, (unsigned)B);
    const dim3 cgrid((unsigned)ly.Hq, (unsigned)B);
    pod_cache *mc = const_cast<pod_cache *>(c);
    const bool prof = mc->prof_ev && mc->prof_n < mc->prof_cap;
    if (prof) POD_HIP_TRY(hipEventRecord(mc->prof_ev[2 * mc->prof_n], st));
#define POD_LAUNCH_PARTIAL(DD, MM, GRID) hipLaunchKernelGGL((decode_partial_kernel<DD, MM>), GRID, dim3(kWaves * 64), 0, st, p)
    // gated upper layer: proximal chunks first, then the distant chunks, whose workgroups read the proximal partials
    const dim3 grid_p((unsigned)(WGS - p.hot.max_nd), (unsigned)ly.Hkv, (unsigned)B);
    const dim3 grid_d((unsigned)(p.hot.max_nd > 0 ? p.hot.max_nd : 1), (unsigned)ly.Hkv, (unsigned)B);
    // score reuse: the writing launch for the kv heads whose block starts at this layer, the reading launch(es) for
    // the others (workgroups of the other kind leave at once); a gated read is two launches, proximal chunks first
#define POD_LAUNCH_ALL(DD)                                                                   \
    if (reuse_step) {                                                                        \
        if (lowest_any) {                                                                    \
            if (fuse == 2 && loc) hipLaunchKernelGGL((decode_partial_kernel<DD, 1, 2, true>), grid, dim3(fuse_waves(2) * 64), 0, st, p); \
            else if (fuse == 2) hipLaunchKernelGGL((decode_partial_kernel<DD, 1, 2>), grid, dim3(fuse_waves(2) * 64), 0, st, p);         \
            else hipLaunchKernelGGL((decode_partial_kernel<DD, 1, 3>), grid, dim3(kWaves * 64), 0, st, p);                               \
        }                                                                                    \
        if (!lowest_all) {                                                                   \
            if (fuse == 2 && loc) hipLaunchKernelGGL((decode_partial_kernel<DD, 2, 2, true>), grid, dim3(fuse_waves(2) * 64), 0, st, p); \
            else if (fuse == 2) hipLaunchKernelGGL((decode_partial_kernel<DD, 2, 2>), grid, dim3(fuse_waves(2) * 64), 0, st, p);         \
            else hipLaunchKernelGGL((decode_partial_kernel<DD, 2, 3>), grid, dim3(kWaves * 64), 0, st, p);                               \
        }                                                                                    \
    }                                                                                        \
    else if (fuse == 2 && loc) hipLaunchKernelGGL((decode_partial_kernel<DD, 0, 2, true>), grid, dim3(fuse_waves(2) * 64), 0, st, p); \
    else if (fuse == 1 && loc) hipLaunchKernelGGL((decode_partial_kernel<DD, 0, 1, true>), grid, dim3(fuse_waves(1) * 64), 0, st, p); \
    else if (fuse == 2) hipLaunchKernelGGL((decode_partial_kernel<DD, 0, 2>), grid, dim3(fuse_waves(2) * 64), 0, st, p);    \
    else if (fuse == 3) hipLaunchKernelGGL((decode_partial_kernel<DD, 0, 3>), grid, dim3(kWaves * 64), 0, st, p);               \
    else if (fuse == 1) hipLaunchKernelGGL((decode_partial_kernel<DD, 0, 1>), grid, dim3(fuse_waves(1) * 64), 0, st, p);    \
    else if (p.mode == 0) POD_LAUNCH_PARTIAL(DD, 0, grid);                                   \
    else {                                                                                   \
        if (lowest_any) POD_LAUNCH_PARTIAL(DD, 1, grid);                                     \
        if (!lowest_all && p.mode == 2) POD_LAUNCH_PARTIAL(DD, 2, grid);                     \
        if (!lowest_all && p.mode == 3) {                                                    \
            POD_LAUNCH_PARTIAL(DD, 3, grid_p);                                               \
            if (p.hot.max_nd > 0) POD_LAUNCH_PARTIAL(DD, 4, grid_d);                         \
        }                                                                                    \
    }
    if (even) {
        const dim3 egrid((unsigned)p.bal_nwg + (step ? (unsigned)npairs : 0u));
#define POD_LAUNCH_EVEN(DD)                                                                                                   \
        if (even_mode == 2) hipLaunchKernelGGL((decode_even_kernel<DD, true, 2>), egrid, dim3(kWaves * 64), 0, st, p);    \
        else if (step) hipLaunchKernelGGL((decode_even_kernel<DD, true, 0>), egrid, dim3(kWaves * 64), 0, st, p);              \
        else hipLaunchKernelGGL((decode_even_kernel<DD, false, 0>), egrid, dim3(kWaves * 64), 0, st, p);
        if (ly.D == 128) { POD_LAUNCH_EVEN(128) } else { POD_LAUNCH_EVEN(64) }
#undef POD_LAUNCH_EVEN
    }
    else if (ly.D == 128) { POD_LAUNCH_ALL(128) } else { POD_LAUNCH_ALL(64) }
#undef POD_LAUNCH_ALL
#undef POD_LAUNCH_PARTIAL
    if (prof) { POD_HIP_TRY(hipEventRecord(mc->prof_ev[2 * mc->prof_n + 1], st)); mc->prof_n += 1; }
    if (fuse == 0 || fuse == 3) {
        if (ly.D == 128)
            hipLaunchKernelGGL((decode_combine_kernel<128, 256, 8, 64>), dim3(cgrid.x, cgrid.y, 2), dim3(256), 0, st, p);
        else
            hipLaunchKernelGGL((decode_combine_kernel<64, 256, 8, 32>), dim3(cgrid.x, cgrid.y, 2), dim3(256), 0, st, p);
    }
    POD_HIP_TRY(hipGetLastError());
    return POD_OK;
}
