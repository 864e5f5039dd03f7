// Prefill attention for PoD: causal flash attention on bf16 MFMA with two logit sources.
//
// For query i and key j <= i (Eq. 3 of the paper with the window taken at the query's own
// position): j is proximal if j < S or j > i - W and its logit is q_l[i].k_l[j]; otherwise it is
// distant and its logit is the block's lowest layer's, q_a[i].k_a[j].  One softmax over all
// j <= i (Eq. 4 / appendix), values always v_l.
//
// Because a softmax accumulates in any order, the key loop runs in two phases, each with ONE
// query operand in registers and ONE key source:
//   phase D (upper layers only): key tiles that hold a distant key for some row of the
//            workgroup, with q_a and k_a; elements that are not distant for their row are masked;
//   phase P: sink tiles and band tiles, with q_l and k_l; elements that are not proximal (or not
//            causal) are masked.
// A tile that straddles a region edge is visited by both phases with complementary masks (its V
// tile is loaded twice: ~4 of 256 tiles per row block at the paper's window sizes).  At the
// block's lowest layer there is only phase P over all tiles, with the causal mask.
//
// Tiling: a workgroup of 4 waves takes 128 query rows of one head, 32 rows per wave; key/value
// tiles of 64 tokens go through LDS.
//   S^T[key][row] = K[key][:] . Q[row][:]     v_mfma_f32_32x32x16_bf16, A = K fragment, B = Q
//   O^T[dim][row] = sum_key V[key][dim] P[key][row]               A = V^T fragment, B = P
// Query row = MFMA column (lane % 32) in both, so softmax state, P and the output slice of a
// row stay in the same lane, and the S^T accumulators become the P operand without moving: the
// 8 keys a lane holds for one PV k-step are the keys of its 8 consecutive accumulators (tokens
// 16 ks + 4 (lane / 32) + {0..3} and + 8 of the tile), and the V^T fragments are read for that order.
//
// Softmax: base-2 with the logit scale folded into the exponent; the reference maximum is only
// moved when a tile exceeds it by more than 2^8 (probabilities then stay below 256, harmless in
// fp32 sums and in bf16), which removes most rescaling passes over the output accumulators.
#include <stdlib.h>
#include <mutex>
#include <type_traits>
#include <utility>

#include "pod_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

constexpr int kBN = 64;
constexpr float kNegBig = -1.0e30f;
constexpr int kPF = 2;        // LDS fragment reads in flight ahead of the MFMA that uses them (1 is slower, 3 no faster)
constexpr float kLazy = 8.0f; // how far (log2) a tile's maximum may exceed the reference before rescaling

struct prefill_params {
    int n, Hq, Hkv, rep, S, W;
    int q0; // position of the first query row: q, qs and out hold rows q0 .. n-1 (k, v, ks hold 0 .. n-1)
    const pod_bf16 *q, *k, *v, *qs, *ks; // qs/ks NULL: own q,k serve every key
    pod_bf16 *out;
    float scale_log2e;
    unsigned long long lowest_mask; // bit h: kv head h takes every logit from (q, k) even if qs/ks are given
    // TAB kernels: k, v, ks are not used.  tile_tab[(stream * Hkv + kv head) * ntiles + key tile] is the device
    // address of that tile's first row for that head, rows D * 2 bytes apart; stream 0 = k, 1 = v, 2 = ks
    const unsigned long long *tile_tab;
    int ntiles;
    // TAB kernels also finish the cache update that wrote the table: if *len still is len_old it becomes len_new,
    // else *flag is raised (the update kernel made the same test and stored nothing)
    int *len, *flag;
    int len_old, len_new;
};

__device__ inline bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ inline unsigned pack_bf16(float lo, float hi)
{
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    bf16x2 t = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(unsigned, t);
}

// Exchange between the two lanes (l, l ^ 32) that share a query row: v_permlane32_swap gives
// lane l its partner's value in one of the two results.  Operands and results go through empty
// asm statements: given the same value twice the compiler otherwise folds max(r0, r1) to r0.
__device__ inline void pair_exchange(float x, float &mine_or_partner0, float &mine_or_partner1)
{
    unsigned a = __builtin_bit_cast(unsigned, x), b = a;
    asm volatile("" : "+v"(b));
    const auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
    unsigned r0 = r[0], r1 = r[1];
    asm volatile("" : "+v"(r0), "+v"(r1)); // (the two results are not interchangeable either)
    mine_or_partner0 = __builtin_bit_cast(float, r0);
    mine_or_partner1 = __builtin_bit_cast(float, r1);
}
__device__ inline float pair_max(float x)
{
    float a, b;
    pair_exchange(x, a, b);
    return fmaxf(a, b);
}
__device__ inline float pair_sum(float x)
{
    float a, b;
    pair_exchange(x, a, b);
    return a + b;
}

// ---------------------------------------------------------------------------------------------
// Order of work inside a wave (software pipeline over three tiles).
//
// Measured on gfx950: a wave issues roughly one vector instruction per 5-6 cycles, a 32x32x16
// MFMA keeps the matrix pipe busy for 32 cycles, and with two waves per SIMD the pipe only
// stays busy if each wave brings at most ~3 ordinary vector instructions, one transcendental
// and one or two LDS reads per MFMA.  So an iteration is a sequence of MFMA slots of that shape,
// taken from three different tiles:
//   iteration t:  S(t+1) = K(t+1) Q^T        (logits of the next tile)
//                 O += V(t-1)^T P(t-1)       (output update of the previous tile)
//                 P(t) = exp2(c S(t) - m)    one pair of elements per slot or two
//                 row maximum of S(t+1); one barrier.
// No exponential waits for an MFMA of the same iteration.  Slot order: the 2:1 mix QK, QK, PV
// for the first three quarters of the slots (all of S(t+1) is then complete), PV only in the
// last quarter, where the vector work is the row maximum of S(t+1).  It is needed at the top of
// the next iteration, which moves the reference maximum if the tile exceeds it by more than 2^8
// and rescales the accumulators (rare).  Masked logits are -infinity (exponential 0 whatever the
// reference); every wave walks every tile of its workgroup.  The row sum adds the bf16-rounded
// probabilities (v_dot2c_f32_bf16 with ones), i.e. exactly the weights the PV product uses.
//
// Data movement uses no registers: K and V tiles go from global memory straight into LDS
// (global_load_lds_dwordx4: each wave instruction fills 1 KB of consecutive LDS, lane l its 16
// bytes; which 16 bytes of the tile a lane fetches is free to choose).
// Both slots are row-major [64 tokens][D] as in global memory, so a wave instruction fetches whole
// rows (256 consecutive bytes per row at D = 128: fully coalesced requests); only the order of the
// 16-byte pieces inside a row is permuted, differently for the two readers:
//   K slot: piece c of row r sits at piece c ^ krot(r), krot(r) = (r D / 128) mod (D / 8).  The B
//           operand of the QK product (one key row, 8 dims per lane) is one ds_read_b128; the 16 rows
//           that such a read touches at once hit 16 different 16-byte bank groups.
//   V slot: 16-byte pieces of a row XOR-permuted by
//           4 (token % 4).  The A operand of the PV product (V^T: one dim, 8 tokens per lane) comes
//           out of two ds_read_b64_tr_b16 (the LDS transpose read: inside 16 lanes, lane L receives
//           element L % 4 of the four 8-byte rows addressed by lanes L / 4 + {0, 4, 8, 12}).
// K(t+2) and V(t) are requested at the top of iteration t into the slots freed by the barrier
// before, and awaited (vmcnt) before the barrier that ends the iteration.
// static_for<N>(f): f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>), each call its own
// instantiation with a compile-time index (no reliance on the loop unroller for big bodies)
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

__device__ inline float dot2_ones(unsigned pk, float acc)
{
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk), ones, acc, false);
}

template <int D, bool TAB>
__global__ __launch_bounds__(256, 2) void prefill_kernel(prefill_params p)
{
    constexpr int CPR = D / 8, KST = D / 16, NDB = D / 32, NKB = kBN / 32, NPS = kBN / 16;
    constexpr int BM = 128;
    constexpr int NQK = NKB * KST;   // MFMAs of one S tile = K fragments of a tile
    constexpr int NPV = NDB * NPS;   // MFMAs of one PV tile (equal to NQK)
    static_assert(NQK == NPV, "slot schedule assumes as many QK as PV MFMAs per tile");
    typedef const __attribute__((address_space(1))) u32x4 *gvec_ptr;
    typedef const __attribute__((address_space(1))) char *gbyte_ptr;
    typedef __attribute__((address_space(3))) char *lbyte_ptr;
    typedef __attribute__((ext_vector_type(4))) short s16x4;
    typedef __attribute__((address_space(3))) s16x4 *ltr_ptr;
    constexpr int FRAG = 64 * 16;
    constexpr int KBUF = NQK * FRAG, VBUF = kBN * D * 2; // 16 KB each at D = 128
    extern __shared__ __attribute__((aligned(16))) char lds[];   // [K slot 0][K slot 1][V slot 0][V slot 1]
    char *const ldsK = lds, *const ldsV = lds + 2 * KBUF;

    const int nqt = (p.n + BM - 1) / BM;
    const int wg = blockIdx.x;
    const int kvh = wg % p.Hkv;
    const int rest = wg / p.Hkv;
    const int head = kvh * p.rep + rest % p.rep;
    // (Query tiles are handed out from the last, which has most keys, to the first.  Which tiles share a CU does not
    // matter: a workgroup takes about as long per key tile alone on its CU as next to a second one, so a launch of
    // one round takes as long as its longest tile either way; pairing long tiles with short ones measured no gain.)
    const int qt = nqt - 1 - rest / p.rep;
    const int i0 = qt * BM;
    const int i_last = min(i0 + BM, p.n) - 1;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n32 = lane & 31, jj = lane >> 5;
    const int iw0 = i0 + wave * 32;
    const int iw_last = min(iw0 + 32, p.n) - 1;
    const int irow = iw0 + n32;
    const bool has_shared = p.qs != nullptr && !((p.lowest_mask >> kvh) & 1);
    const int S = p.S, W = p.W;
    const float c = p.scale_log2e;

    int tD0 = 0, nD = 0, nP1 = 0, tB = 0;
    if (has_shared) {
        if (i_last - W >= S) { tD0 = S / kBN; nD = (i_last - W) / kBN - tD0 + 1; }
        if (S > 0) nP1 = (min(S, i_last + 1) - 1) / kBN + 1;
        tB = max(nP1, max(0, i0 - W + 1) / kBN);
    }
    const int tEnd = i_last / kBN;
    const int nP2 = tEnd >= tB ? tEnd - tB + 1 : 0;
    const int T = nD + nP1 + nP2;
    auto tile_of = [&](int t, int &kt, bool &phaseD) {
        phaseD = t < nD;
        kt = phaseD ? tD0 + t : (t < nD + nP1 ? t - nD : tB + (t - nD - nP1));
    };

    // ---- global -> LDS.  Wave w moves K fragments w*NQK/4 .. and the V rows w*16 .. w*16+15.
    constexpr int VRI = 64 / CPR;                // V rows per wave instruction (1 KB)
    constexpr int VPW = 16 / VRI;                // V instructions per wave and tile
    constexpr int VSWZ = 4 * ((CPR / 4 - 1) & 3); // piece-permutation mask: 12 at D = 128, 4 at D = 64
    // A request is ONE scalar base per tile plus a per-lane offset that never changes (one register per
    // request of the wave), so a tile costs neither vector nor scalar address arithmetic; only the
    // prompt's last, partly filled tile takes a separate path that clamps its rows per lane.
    const unsigned rowb = TAB ? (unsigned)(D * 2) : (unsigned)p.Hkv * D * 2; // TAB: one head's rows, back to back
    const unsigned head_col = TAB ? 0u : (unsigned)(kvh * D * 2);
    typedef const __attribute__((address_space(4))) unsigned long long *tab_ptr;  // read with scalar loads
    const tab_ptr tab_k = (tab_ptr)(p.tile_tab + (size_t)kvh * p.ntiles);
    const size_t tab_stream = (size_t)p.Hkv * p.ntiles;
    const int v_r = lane / CPR;                                         // row inside a V instruction
    // K rows: a lane of a request fetches piece (slot piece ^ krot(row)) of its row, krot(row) = row * CPR / 16 mod CPR
    // (16 consecutive rows then put the same piece into 16 different 16-byte bank groups)
    auto k_col = [&](int x) { // x-th request of the wave: LDS rows 16 wave + VRI x + v_r
        const int rot = (((VRI * x + v_r) * CPR) / 16) & (CPR - 1);
        return head_col + (unsigned)(16 * ((lane % CPR) ^ rot));
    };
    const unsigned v_col = head_col + (unsigned)(16 * ((lane % CPR) ^ ((4 * (v_r & 3)) & VSWZ)));
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);            // scalar copy: LDS destinations stay scalar
    unsigned k_off[VPW], v_off[VPW];
#pragma unroll
    for (int x = 0; x < VPW; ++x) {
        v_off[x] = (unsigned)(16 * wave + VRI * x + v_r) * rowb + v_col;
        k_off[x] = (unsigned)(16 * wave + VRI * x + v_r) * rowb + k_col(x);
    }
    typedef const __attribute__((address_space(1))) void *gvoid_ptr;
    typedef __attribute__((address_space(3))) void *lvoid_ptr;
    const char *const k_dst0 = ldsK + wave_s * (16 * D * 2);            // this wave's part of K slot 0
    const char *const v_dst0 = ldsV + wave_s * (16 * D * 2);            // this wave's part of V slot 0
    // TAB: the tile's address comes out of the table with a scalar load; the callers fetch it an iteration ahead
    auto k_tile = [&](int kt, bool phaseD) { return tab_k[(phaseD ? 2 * tab_stream : 0) + kt]; };
    auto v_tile = [&](int kt) { return tab_k[tab_stream + kt]; };
    auto request_k = [&](int kt, bool phaseD, int slot, unsigned long long tile) {
        const int j0 = kt * kBN;
        gbyte_ptr base;
        if constexpr (TAB) base = (gbyte_ptr)tile;
        else base = (gbyte_ptr)(phaseD ? p.ks : p.k) + (size_t)j0 * rowb;
        if (__builtin_expect(j0 + kBN <= p.n, 1)) {
#pragma unroll
            for (int x = 0; x < VPW; ++x) {
                unsigned off = k_off[x];
                asm volatile("" : "+v"(off)); // (else the compiler keeps 64-bit copies of all offsets live: 8 more registers)
                __builtin_amdgcn_global_load_lds((gvoid_ptr)(base + off), (lvoid_ptr)(k_dst0 + slot * KBUF + x * (VRI * D * 2)), 16, 0, 0);
            }
        } else {
            asm volatile("" ::: "memory"); // (keeps this a real branch: merged, both paths would pay for the clamping)
#pragma unroll
            for (int x = 0; x < VPW; ++x) {
                const unsigned off = (unsigned)min(16 * wave + VRI * x + v_r, p.n - 1 - j0) * rowb + k_col(x);
                __builtin_amdgcn_global_load_lds((gvoid_ptr)(base + off), (lvoid_ptr)(k_dst0 + slot * KBUF + x * (VRI * D * 2)), 16, 0, 0);
            }
        }
    };
    auto request_v = [&](int kt, int slot, unsigned long long tile) {
        const int j0 = kt * kBN;
        gbyte_ptr base;
        if constexpr (TAB) base = (gbyte_ptr)tile;
        else base = (gbyte_ptr)p.v + (size_t)j0 * rowb;
        if (__builtin_expect(j0 + kBN <= p.n, 1)) {
#pragma unroll
            for (int x = 0; x < VPW; ++x) {
                unsigned off = v_off[x];
                asm volatile("" : "+v"(off));
                __builtin_amdgcn_global_load_lds((gvoid_ptr)(base + off), (lvoid_ptr)(v_dst0 + slot * VBUF + x * (VRI * D * 2)), 16, 0, 0);
            }
        } else {
            asm volatile("" ::: "memory");
#pragma unroll
            for (int x = 0; x < VPW; ++x) {
                const unsigned off = (unsigned)min(16 * wave + VRI * x + v_r, p.n - 1 - j0) * rowb + v_col;
                __builtin_amdgcn_global_load_lds((gvoid_ptr)(base + off), (lvoid_ptr)(v_dst0 + slot * VBUF + x * (VRI * D * 2)), 16, 0, 0);
            }
        }
    };
    // read offsets: K fragment lane slot; V^T transpose-read source row/piece of this lane
    // K fragment (key block kb, k-step s): lane (row n32, jj) reads piece 2 s + jj of row 32 kb + n32, stored at
    // piece (2 s + jj) ^ krot(row) = (jj ^ krot) ^ 2 s; krot(32 kb + n32) = krot(n32)
    const int k_rot = ((n32 * CPR) / 16) & (CPR - 1);
    const int k_rd0 = n32 * (D * 2) + 16 * (jj ^ k_rot);
    const int v_s = lane & 15;
    // row 4 jj + s/4 of the 16-token k-step (+8 for the second read), dims 16 ((lane/16) & 1) + 4 (s % 4) of the
    // 32-dim block db; the piece index is XORed with 4 (row % 4) = 4 (s / 4), the dim block enters as XOR 64 db
    const int v_rd0 = (4 * jj + (v_s >> 2)) * (D * 2) + ((64 * (v_s >> 2)) & (16 * VSWZ)) + 32 * ((lane >> 4) & 1) + 8 * (v_s & 3);
    int v_rd[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db) v_rd[db] = v_rd0 ^ (64 * db);

    bf16x8 qf[KST];
    const int qrow = max(min(irow, p.n - 1), p.q0) - p.q0;
    auto load_q = [&](const pod_bf16 *src) {
        const gvec_ptr qr = (gvec_ptr)(src + ((size_t)qrow * p.Hq + head) * D);
#pragma unroll
        for (int s = 0; s < KST; ++s) qf[s] = as_bf16x8(qr[2 * s + jj]);
    };

    // -infinity on the logits of key block kb of tile (kt, phase) that are not this phase's to count
    auto mask_block = [&](int kt, bool phaseD, int kb, f32x16 &sc) {
        const int j0 = kt * kBN;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int j = j0 + 32 * kb + 8 * (r >> 2) + 4 * jj + (r & 3);
            const bool okD = (j >= S) & (j <= irow - W);
            const bool okP = (j <= irow) & ((!has_shared) | (j < S) | (j > irow - W));
            const bool ok = phaseD ? okD : okP;
            sc[r] = ok ? sc[r] : -__builtin_inff();
        }
    };
    auto mask_tile = [&](int kt, bool phaseD, f32x16 (&sc)[NKB]) {
        const int j0 = kt * kBN, j1 = j0 + kBN - 1;
        bool full; // every (row, key) pair of the wave counts: no masking needed
        if (phaseD) full = j0 >= S && j1 <= iw0 - W;
        else if (has_shared) full = j1 <= iw0 && (j1 < S || j0 > iw_last - W);
        else full = j1 <= iw0;
        if (full && iw0 <= iw_last) return;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) mask_block(kt, phaseD, kb, sc[kb]);
    };

    f32x16 oacc[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
    float m_ref = kNegBig, l_run = 0.f;

    auto kfrag = [&](const char *kl, int op) { // QK MFMA number op: the two key blocks alternate
        const int s = op / NKB, kb = op % NKB;
        return *(const u32x4 *)(kl + kb * 32 * (D * 2) + (k_rd0 ^ (32 * s)));
    };
    auto vfrag = [&](const char *vl, int m) {  // PV MFMA number m = ks * NDB + db
        const int ks = m / NDB, db = m % NDB;
        const lbyte_ptr a = (lbyte_ptr)(vl + ks * 16 * (D * 2)) + v_rd[db];
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ltr_ptr)a);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((ltr_ptr)(a + 8 * (D * 2)));
        u32x4 r;
        const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
        r.x = l2.x; r.y = l2.y; r.z = h2.x; r.w = h2.y;
        return r;
    };

    f32x16 sA[NKB], sB[NKB];
    u32x4 pA[NPS], pB[NPS];
    float mx_next; // scaled row maximum of the tile the next iteration exponentiates

    // ---- prologue: K(0), K(1) in LDS, S(0) and its row maximum computed
    // tiles t, t+1, t+2 of the current iteration (key tile index, phase); shifted along at its end
    int kt_a, kt_b, kt_c;
    bool ph_a, ph_b, ph_c;
    tile_of(0, kt_a, ph_a);
    tile_of(1, kt_b, ph_b);
    tile_of(2, kt_c, ph_c);
    unsigned long long k_next = 0, v_next = 0; // TAB: addresses of the tiles the next iteration requests
    if constexpr (TAB) {
        if (wg == 0 && tid == 0) { // the update launch before this one left the length for here
            if (*p.len == p.len_old) *p.len = p.len_new;
            else atomicOr(p.flag, 1);
        }
        request_k(kt_a, ph_a, 0, k_tile(kt_a, ph_a));
        if (T > 1) request_k(kt_b, ph_b, 1, k_tile(kt_b, ph_b));
        if (T > 2) k_next = k_tile(kt_c, ph_c);
        v_next = v_tile(kt_a);
    } else {
        request_k(kt_a, ph_a, 0, 0);
        if (T > 1) request_k(kt_b, ph_b, 1, 0);
    }
    load_q(nD > 0 ? p.qs : p.q);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    {
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) sA[kb][r] = 0.f;
#pragma unroll
        for (int op = 0; op < NQK; ++op) {
            const int s = op / NKB, kb = op % NKB;
            sA[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kfrag(ldsK, op)), qf[s], sA[kb], 0, 0, 0);
        }
        mask_tile(kt_a, ph_a, sA);
        float mx = -__builtin_inff();
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sA[kb][r]);
        mx_next = pair_max(mx) * c;
    }
    __syncthreads(); // every wave is done reading K(0): iteration 0 overwrites its slot

    // one iteration: FIRST has no PV slots (there is no earlier tile)
    auto iteration = [&](auto first_tag, auto slot_tag, int t, f32x16 (&sc)[NKB], f32x16 (&sn)[NKB], u32x4 (&pprev)[NPS], u32x4 (&pcur)[NPS]) {
        constexpr bool FIRST = decltype(first_tag)::value;
        constexpr int slot = decltype(slot_tag)::value; // = t % 2: every LDS address below is a compile-time offset
        // K(t+2) replaces K(t) and V(t) replaces V(t-2), both last read before the previous barrier.
        // (Spreading the requests over the slots instead of issuing them here measured 10 % slower.)
        if (t + 2 < T) request_k(kt_c, ph_c, slot, k_next);
        request_v(kt_a, slot, v_next);
        if constexpr (TAB) {
            int kt_d; bool ph_d;
            tile_of(t + 3, kt_d, ph_d);
            if (t + 3 < T) k_next = k_tile(kt_d, ph_d);
            if (t + 1 < T) v_next = v_tile(kt_b);
        }
        if (mx_next > m_ref + kLazy) { // (rows with nothing valid so far have mx = -inf and never trigger)
            // The reference moves before tile t is exponentiated: everything computed with the old one is brought
            // to the new one.  That is the row sum, the output accumulators (tiles <= t-2), and P(t-1), whose
            // product with V(t-1) is still to come in this iteration's PV slots.
            const float alpha = __builtin_amdgcn_exp2f(m_ref - mx_next);
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
            if constexpr (!FIRST) {
#pragma unroll
                for (int ks = 0; ks < NPS; ++ks)
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        const unsigned pk = pprev[ks][w];
                        const float lo = __builtin_bit_cast(float, pk << 16), hi = __builtin_bit_cast(float, pk & 0xffff0000u);
                        pprev[ks][w] = pack_bf16(lo * alpha, hi * alpha);
                    }
            }
            m_ref = mx_next;
        }
        if (t + 1 == nD) load_q(p.q); // the next tile is the first of the own-key phase
        const float mr = m_ref;
        float ps = 0.f;
        const char *kl = ldsK + (slot ^ 1) * KBUF;   // K(t+1)
        const char *vl = ldsV + (slot ^ 1) * VBUF;   // V(t-1)
        // slot list: entry >= 0 is QK MFMA number entry, entry < 0 is PV MFMA number -1 - entry
        constexpr int NS = FIRST ? NQK : NQK + NPV;
        constexpr int NMIX = FIRST ? NQK : NQK + NQK / 2; // slots of the QK, QK, PV mix
        auto slot_op = [](int i) constexpr { return FIRST ? i : (i < NMIX ? ((i % 3 == 2) ? -1 - i / 3 : i - i / 3) : -1 - (i - NQK)); };
        auto frag = [&](int i) { const int op = slot_op(i); return op >= 0 ? kfrag(kl, op) : vfrag(vl, -1 - op); };
        u32x4 fr[NS];
        float tt[16][2], ee[16][2]; // staged softmax values (each lives for one slot)
        float mxv[4] = {-__builtin_inff(), -__builtin_inff(), -__builtin_inff(), -__builtin_inff()};
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < kPF && i < NS; ++i) fr[i] = frag(i);
        static_for<NS>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            if constexpr (!FIRST && i == NMIX) {
                mask_tile(kt_b, ph_b, sn); // boundary tiles only; S(t+1) is complete here
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (i + kPF < NS) fr[i + kPF] = frag(i + kPF);
            constexpr int op = slot_op(i);
            if constexpr (op >= 0) {
                constexpr int s = op / NKB, kb = op % NKB;
                if constexpr (s == 0) {
                    f32x16 z;
#pragma unroll
                    for (int r = 0; r < 16; ++r) z[r] = 0.f;
                    sn[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fr[i]), qf[s], z, 0, 0, 0);
                } else {
                    sn[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fr[i]), qf[s], sn[kb], 0, 0, 0);
                }
            } else {
                constexpr int m = -1 - op, ks = m / NDB, db = m % NDB;
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(fr[i]), as_bf16x8(pprev[ks]), oacc[db], 0, 0, 0);
            }
            if constexpr (i < NMIX) {
                // this slot's share of the 16 logit pairs of tile t.  A pair takes three steps (scale and
                // shift; exponentials; pack and row sum) in three different slots, so that no
                // instruction of a slot waits for another one of the same slot.
                constexpr int v_lo = (i * 18 + NMIX - 1) / NMIX; // first step v with v * NMIX / 18 == i, if any
                static_for<(18 + NMIX - 1) / NMIX + 1>([&](auto dvc) {
                    constexpr int v = v_lo + decltype(dvc)::value;
                    if constexpr (v < 18 && v * NMIX / 18 == i) {
                        if constexpr (v >= 2) {
                            constexpr int q = v - 2;
                            unsigned pk = pack_bf16(ee[q][0], ee[q][1]);
                            ps = dot2_ones(pk, ps);
                            // an empty asm statement is a use the compiler cannot move: without it, work whose
                            // consumer sits in a later basic block is sunk out of the slot it was placed in
                            asm volatile("" : "+v"(pk), "+v"(ps));
                            pcur[q >> 2][q & 3] = pk;
                        }
                        if constexpr (v >= 1 && v <= 16) {
                            constexpr int q = v - 1;
                            float e0 = __builtin_amdgcn_exp2f(tt[q][0]), e1 = __builtin_amdgcn_exp2f(tt[q][1]);
                            asm volatile("" : "+v"(e0), "+v"(e1));
                            ee[q][0] = e0; ee[q][1] = e1;
                        }
                        if constexpr (v <= 15) {
                            constexpr int q = v;
                            float t0 = fmaf(sc[q >> 3][(2 * q) & 15], c, -mr), t1 = fmaf(sc[q >> 3][((2 * q) & 15) + 1], c, -mr);
                            asm volatile("" : "+v"(t0), "+v"(t1));
                            tt[q][0] = t0; tt[q][1] = t1;
                        }
                    }
                });
            } else {
                // last quarter: row maximum of S(t+1)
                constexpr int NL = NS - NMIX, j = i - NMIX;
                constexpr int XPS = NKB * 16 / (NL > 0 ? NL : 1); // logits per slot (FIRST has no such slots)
                static_assert(NL == 0 || (XPS * NL == NKB * 16 && XPS % 2 == 0), "");
#pragma unroll
                for (int x = j * XPS; x < (j + 1) * XPS; x += 2) {
                    float mm = __builtin_fmaxf(__builtin_fmaxf(mxv[(x >> 1) & 3], sn[x >> 4][x & 15]), sn[x >> 4][(x & 15) + 1]);
                    asm volatile("" : "+v"(mm));
                    mxv[(x >> 1) & 3] = mm;
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        if (FIRST) { // no last quarter: the same housekeeping without MFMAs in between
            mask_tile(kt_b, ph_b, sn);
#pragma unroll
            for (int x = 0; x < NKB * 16; ++x) mxv[x & 3] = fmaxf(mxv[x & 3], sn[x >> 4][x & 15]);
        }
        mx_next = pair_max(fmaxf(fmaxf(mxv[0], mxv[1]), fmaxf(mxv[2], mxv[3]))) * c;
        l_run += ps;
        kt_a = kt_b; ph_a = ph_b; kt_b = kt_c; ph_b = ph_c;
        tile_of(t + 3, kt_c, ph_c);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); // this wave's K(t+2), V(t) pieces are in LDS
        __syncthreads();
    };


    typedef std::integral_constant<int, 0> slot0;
    typedef std::integral_constant<int, 1> slot1;
    iteration(std::true_type{}, slot0{}, 0, sA, sB, pB, pA);
    for (int t = 1; t < T; t += 2) {
        iteration(std::false_type{}, slot1{}, t, sB, sA, pA, pB);
        if (t + 1 < T) iteration(std::false_type{}, slot0{}, t + 1, sA, sB, pB, pA);
    }
    // ---- epilogue: O += V(T-1)^T P(T-1)
    {
        const char *vl = ldsV + ((T - 1) & 1) * VBUF;
        auto pv = [&](const u32x4 (&pw)[NPS]) {
#pragma unroll
            for (int m = 0; m < NPV; ++m)
                oacc[m % NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(vfrag(vl, m)), as_bf16x8(pw[m / NDB]), oacc[m % NDB], 0, 0, 0);
        };
        if ((T - 1) & 1) pv(pB);
        else pv(pA);
    }

    const float l = pair_sum(l_run);
    if (irow < p.n && irow >= p.q0) {
        const float inv = 1.f / l;
        pod_bf16 *orow = p.out + ((size_t)(irow - p.q0) * p.Hq + head) * D;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                u32x2 o;
                o.x = pack_bf16(oacc[db][4 * a + 0] * inv, oacc[db][4 * a + 1] * inv);
                o.y = pack_bf16(oacc[db][4 * a + 2] * inv, oacc[db][4 * a + 3] * inv);
                *(u32x2 *)(orow + 32 * db + 8 * a + 4 * jj) = o;
            }
    }
}

} // namespace

// tile_tab != NULL: keys and values are located through the per-tile address table (k, v, k_shared are not read)
static int launch_prefill(const pod_layout &ly, int n, int q0, const void *q, const void *k, const void *v,
                          const void *q_shared, const void *k_shared, const unsigned long long *tile_tab, int ntiles,
                          int *len, int *flag, uint64_t lowest_mask, float scale, void *out, hipStream_t st)
{
    prefill_params p;
    p.n = n; p.q0 = q0; p.Hq = ly.Hq; p.Hkv = ly.Hkv; p.rep = ly.rep; p.S = ly.S; p.W = ly.W;
    p.q = (const pod_bf16 *)q; p.k = (const pod_bf16 *)k; p.v = (const pod_bf16 *)v;
    p.qs = (const pod_bf16 *)q_shared; p.ks = (const pod_bf16 *)k_shared;
    p.out = (pod_bf16 *)out;
    p.scale_log2e = scale * 1.4426950408889634f;
    p.lowest_mask = lowest_mask;
    p.tile_tab = tile_tab; p.ntiles = ntiles;
    p.len = len; p.flag = flag; p.len_old = q0; p.len_new = n;
    if (scale <= 0.f) return pod_fail(POD_ERR_INVALID_ARG, "scale must be positive");
    if (tile_tab && ntiles < (n + kBN - 1) / kBN) return pod_fail(POD_ERR_INVALID_ARG, "tile table of %d entries for %d keys", ntiles, n);
    // query tiles of 128 positions, counted from the end: the kernel takes tile (n + 127) / 128 - 1 - blockIdx.x / Hq
    const dim3 grid((unsigned)((n + 127) / 128 - q0 / 128) * (unsigned)ly.Hq);
    // dynamic LDS: two K slots and two V slots of kBN tokens x D bf16 each (64 KB at D = 128)
    const auto lds_bytes = [](int D) { return 4 * kBN * D * 2; };
    // raising the dynamic-LDS limit to 64 KB is needed once per device; any host thread may get here first
    {
        static std::mutex attr_mutex;
        static bool attr_done[64] = {};
        int dev = -1;
        POD_HIP_TRY(hipGetDevice(&dev));
        if (dev < 0 || dev >= 64) return pod_fail(POD_ERR_INVALID_ARG, "device %d outside [0, 64)", dev);
        std::lock_guard<std::mutex> lock(attr_mutex);
        if (!attr_done[dev]) {
            POD_HIP_TRY(hipFuncSetAttribute((const void *)prefill_kernel<128, false>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(128)));
            POD_HIP_TRY(hipFuncSetAttribute((const void *)prefill_kernel<64, false>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(64)));
            POD_HIP_TRY(hipFuncSetAttribute((const void *)prefill_kernel<128, true>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(128)));
            POD_HIP_TRY(hipFuncSetAttribute((const void *)prefill_kernel<64, true>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(64)));
            attr_done[dev] = true;
        }
    }
    if (ly.D == 128) {
        if (tile_tab) hipLaunchKernelGGL((prefill_kernel<128, true>), grid, dim3(256), lds_bytes(128), st, p);
        else hipLaunchKernelGGL((prefill_kernel<128, false>), grid, dim3(256), lds_bytes(128), st, p);
    } else {
        if (tile_tab) hipLaunchKernelGGL((prefill_kernel<64, true>), grid, dim3(256), lds_bytes(64), st, p);
        else hipLaunchKernelGGL((prefill_kernel<64, false>), grid, dim3(256), lds_bytes(64), st, p);
    }
    POD_HIP_TRY(hipGetLastError());
    return POD_OK;
}

int pod_launch_prefill(const pod_layout &ly, int layer, int n, int q0, const void *q, const void *k, const void *v,
                       const void *q_shared, const void *k_shared, uint64_t lowest_mask, float scale, void *out,
                       hipStream_t st)
{
    (void)layer;
    return launch_prefill(ly, n, q0, q, k, v, q_shared, k_shared, nullptr, 0, nullptr, nullptr, lowest_mask, scale, out, st);
}

int pod_launch_prefill_tiles(const pod_layout &ly, int n, int q0, const void *q, const void *q_shared,
                             const unsigned long long *tile_tab, int ntiles, int *len, int *flag, uint64_t lowest_mask, float scale,
                             void *out, hipStream_t st)
{
    return launch_prefill(ly, n, q0, q, nullptr, nullptr, q_shared, nullptr, tile_tab, ntiles, len, flag, lowest_mask, scale, out, st);
}
