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
// Tiling: a workgroup of 4 waves takes BM = 128*NQ query rows of one head; each wave owns 32*NQ
// rows.  Key/value tiles of BN = 64 tokens go through LDS (double-buffered, one barrier per
// tile), written in MFMA A-operand *fragment order* (64 lanes x 16 bytes per fragment) so that
// every read is one conflict-free ds_read_b128.  Global loads of tile t+1 are issued before the
// arithmetic of tile t and parked in registers.
//   S^T[key][row] = K[key][:] . Q[row][:]     v_mfma_f32_32x32x16_bf16, A = K frag, B = Q
//   O^T[dim][row] = sum_key V[key][dim] P[key][row]               A = V^T frag, B = P
// Query row = MFMA column (lane % 32) in both, so softmax state, P and the output slice of a
// row stay in the same lane, and the S^T accumulators become the P operand without moving
// (the 8 keys a lane holds for one PV k-step are the keys of its 8 consecutive accumulators;
// V^T fragments are built for that key order).  V is transposed on the way into LDS: a thread
// loads the same 16-byte dim piece of 4 tokens and transposes the 4x8 block with v_perm_b32.
//
// Softmax: base-2 with the logit scale folded into the exponent; the running maximum is only
// moved when a tile exceeds it by more than 2^8 (probabilities then stay below 256, harmless in
// fp32 sums and in bf16), which removes most rescaling passes over the output accumulators.
#include <type_traits>

#include "pod_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

constexpr int kBN = 64;
constexpr float kNegBig = -1.0e30f;
constexpr float kLazy = 8.0f; // how far (log2) a tile's maximum may exceed the reference before rescaling

struct prefill_params {
    int n, Hq, Hkv, rep, S, W;
    const pod_bf16 *q, *k, *v, *qs, *ks; // qs/ks NULL: own q,k serve every key
    pod_bf16 *out;
    float scale_log2e;
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

template <int D, int NQ>
__global__ __launch_bounds__(256, NQ == 1 ? 2 : 1) void prefill_kernel(prefill_params p)
{
    constexpr int CPR = D / 8;       // 16-byte pieces per row
    constexpr int KST = D / 16;      // QK k-steps (32x32x16)
    constexpr int NDB = D / 32;      // output dim blocks
    constexpr int NKB = kBN / 32;    // key blocks per tile
    constexpr int NPS = kBN / 16;    // PV k-steps per tile
    constexpr int BM = 128 * NQ;
    constexpr int KIT = kBN * CPR / 256; // K pieces per thread per tile
    typedef const __attribute__((address_space(1))) u32x4 *gvec_ptr;

    // LDS: two buffers, each holding NKB*KST key fragments and NDB*NPS V^T fragments of 64 lane
    // slots x 16 bytes.  Inside a fragment the slot of lane l is l ^ x, where x (3 bits) depends on
    // the fragment and on l / 32 for keys, on l / 8 and the dim block for values: with these XORs
    // the reads (one ds_read_b128 per fragment and wave), the key-row writes and the 8-byte V^T
    // writes were all measured free of bank conflicts on gfx950 (64 banks of 4 bytes).  The read
    // offsets take only 4 (keys) + 2 (values) distinct per-lane values, computed once.
    constexpr int FRAG = 64 * 16;
    constexpr int KSTRIDE = FRAG, VSTRIDE = FRAG;
    constexpr int KBUF = NKB * KST * KSTRIDE, VBUF = NDB * NPS * VSTRIDE;
    constexpr int BUF = KBUF + VBUF;           // one buffer: keys then values
    extern __shared__ __attribute__((aligned(16))) char lds[];

    // Workgroup -> (kv head, query head of the group, row block).  Consecutive workgroup ids land
    // on consecutive XCDs (8 of them, each with its own L2), so the kv head is taken from the low
    // bits of the id: with 8 kv heads every XCD works on ONE kv head, and the workgroups resident
    // on it (the 4 query heads of the group x neighbouring row blocks) stream the same K/V tiles
    // at the same time and share them through that L2.  Heaviest row blocks first.
    const int nqt = (p.n + BM - 1) / BM;
    const int wg = blockIdx.x;
    const int kvh = wg % p.Hkv;
    const int rest = wg / p.Hkv;
    const int head = kvh * p.rep + rest % p.rep;
    const int qt = nqt - 1 - rest / p.rep;
    const int i0 = qt * BM;
    const int i_last = min(i0 + BM, p.n) - 1;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n32 = lane & 31, jj = lane >> 5;
    int kroff[4], vroff[2];                          // read offsets of this lane inside a key / value fragment
#pragma unroll
    for (int x = 0; x < 4; ++x) kroff[x] = 16 * (lane ^ (x | (jj << 2)));
#pragma unroll
    for (int x = 0; x < 2; ++x) vroff[x] = 16 * (lane ^ (((lane >> 3) & 3) | (((lane >> 5) ^ x) << 2)));
    const int iw0 = i0 + wave * 32 * NQ;             // first row of this wave
    const int iw_last = min(iw0 + 32 * NQ, p.n) - 1; // may be < iw0: the wave has no rows
    const bool has_shared = p.qs != nullptr;
    const int S = p.S, W = p.W;

    // ---- the tile schedule of this workgroup: nD distant-phase tiles, then sink tiles, then band tiles
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

    // ---- global -> register loads of one tile.  Row addresses are a per-tile scalar base plus ONE
    // per-thread offset (for K and for V), so a tile costs no vector address arithmetic; only the
    // prompt's last, partly filled tile clamps rows to n-1 per thread.
    constexpr int RS = 256 / CPR;                               // key rows covered by one K load of the workgroup
    const int kc = tid % CPR, kr0 = tid / CPR;                  // K: piece, first row
    const int vrest = tid / CPR;                                // V: 4-token group of this thread
    const bool vact = vrest < 16;
    const int vhalf = vrest & 1, vj = (vrest >> 1) & 1, vku = vrest >> 2;
    const int vrow0 = 16 * vku + 8 * vhalf + 4 * vj;            // first of this thread's 4 V rows in the tile
    const unsigned rowb = (unsigned)p.Hkv * D * 2;              // bytes from one token to the next
    const unsigned koff = (unsigned)kr0 * rowb + (unsigned)(kvh * D * 2 + kc * 16);
    const unsigned voff = (unsigned)vrow0 * rowb + (unsigned)(kvh * D * 2 + kc * 16);
    typedef const __attribute__((address_space(1))) char *gbyte_ptr;
    u32x4 kreg[KIT], vreg[4];
    auto load_tile = [&](int t) {
        int kt; bool phaseD;
        tile_of(t, kt, phaseD);
        const int j0 = kt * kBN;
        const gbyte_ptr kb = (gbyte_ptr)(phaseD ? p.ks : p.k) + (size_t)j0 * rowb;
        const gbyte_ptr vb = (gbyte_ptr)p.v + (size_t)j0 * rowb;
        if (j0 + kBN <= p.n) {
#pragma unroll
            for (int it = 0; it < KIT; ++it) kreg[it] = *(gvec_ptr)(kb + (size_t)(it * RS) * rowb + koff);
            if (vact) {
#pragma unroll
                for (int e = 0; e < 4; ++e) vreg[e] = *(gvec_ptr)(vb + (size_t)e * rowb + voff);
            }
        } else {
            const unsigned colb = (unsigned)(kvh * D * 2 + kc * 16);
#pragma unroll
            for (int it = 0; it < KIT; ++it) {
                const int key = min(kr0 + RS * it, p.n - 1 - j0);
                kreg[it] = *(gvec_ptr)(kb + (size_t)key * rowb + colb);
            }
            if (vact) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int key = min(vrow0 + e, p.n - 1 - j0);
                    vreg[e] = *(gvec_ptr)(vb + (size_t)key * rowb + colb);
                }
            }
        }
    };
    // register -> LDS: K pieces into fragment (kb, s = kc/2), slot (row % 32) + 32*(kc % 2); V pieces
    // transposed (4 tokens x 8 dims -> 8 dims x 4 tokens) into fragment (db, ks), slot (dim % 32) + 32*vj.
    // (the XOR only touches the low 3 slot bits, which the +16-row and +dim steps below leave alone)
    const int kw_base = (kc >> 1) * KSTRIDE + 16 * ((kr0 + 32 * (kc & 1)) ^ (((kc >> 1) & 3) | ((kc & 1) << 2)));
    const int vw_x = (kc & 3) | ((vj ^ ((kc >> 2) & 1)) << 2);   // XOR term of this thread's V^T slots
    const int vw_base = KBUF + ((kc >> 2) * NPS + vku) * VSTRIDE + 16 * (8 * (kc & 3) + 32 * vj) + 8 * vhalf;
    auto store_tile = [&](int buf) {
        char *base = lds + buf * BUF;
#pragma unroll
        for (int it = 0; it < KIT; ++it) {
            const int kbk = (RS * it) >> 5, radd = (RS * it) & 31;  // key block, row offset inside it (0 or 16)
            *(u32x4 *)(base + kw_base + kbk * KST * KSTRIDE + 16 * radd) = kreg[it];
        }
        if (vact) {
#pragma unroll
            for (int dlt = 0; dlt < 8; ++dlt) {
                const unsigned sel = (dlt & 1) ? 0x07060302u : 0x05040100u;
                u32x2 pk;
                pk.x = __builtin_amdgcn_perm(vreg[1][dlt >> 1], vreg[0][dlt >> 1], sel);
                pk.y = __builtin_amdgcn_perm(vreg[3][dlt >> 1], vreg[2][dlt >> 1], sel);
                *(u32x2 *)(base + vw_base + 16 * (dlt ^ vw_x)) = pk;
            }
        }
    };

    // ---- query operand of the current phase: lane (row n32, jj) holds dims 16s + 8jj .. +7
    bf16x8 qf[NQ][KST];
    auto load_q = [&](const pod_bf16 *src) {
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
            const int row = min(iw0 + 32 * nq + n32, p.n - 1);
            const gvec_ptr qr = (gvec_ptr)(src + ((size_t)row * p.Hq + head) * D);
#pragma unroll
            for (int s = 0; s < KST; ++s) qf[nq][s] = as_bf16x8(qr[2 * s + jj]);
        }
    };

    f32x16 oacc[NQ][NDB];
    float m_ref[NQ], l_run[NQ]; // l_run: this lane's keys only; the two lanes of a row are added at the end
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        m_ref[nq] = kNegBig; l_run[nq] = 0.f;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[nq][db][r] = 0.f;
    }

    if (T > 0) {
        load_tile(0);
        load_q(nD > 0 ? p.qs : p.q);
        store_tile(0);
        if (T > 1) load_tile(1); // stays in registers while tile 0 is processed
    }
    __syncthreads();

    for (int t = 0; t < T; ++t) {
        const int buf = t & 1;
        int kt; bool phaseD;
        tile_of(t, kt, phaseD);
        if (t == nD && nD > 0) load_q(p.q); // phase switch: own queries from here on

        const int j0 = kt * kBN, j1 = j0 + kBN - 1;
        // does this wave have anything in the tile, and is every (row, key) pair of it valid?
        bool any, full;
        if (phaseD) {
            any = j0 <= iw_last - W && j1 >= S;
            full = j0 >= S && j1 <= iw0 - W;
        } else if (has_shared) {
            any = j0 <= iw_last && (j0 < S || j1 > iw0 - W);
            full = j1 <= iw0 && (j1 < S || j0 > iw_last - W);
        } else {
            any = j0 <= iw_last;
            full = j1 <= iw0;
        }
        // The arithmetic of one tile, compiled twice: FULL = every (row, key) pair of the wave is
        // valid (no mask arithmetic at all) and the general case with the per-element predicate.
        auto tile_body = [&](auto full_tag) {
            constexpr bool FULL = decltype(full_tag)::value;
            const char *lbuf = lds + buf * BUF;
            // ---- S^T = K Q^T
            f32x16 sc[NQ][NKB];
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
                for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) sc[nq][kb][r] = 0.f;
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
                for (int s = 0; s < KST; ++s) {
                    const u32x4 a = *(const u32x4 *)(lbuf + (kb * KST + s) * KSTRIDE + kroff[s & 3]);
#pragma unroll
                    for (int nq = 0; nq < NQ; ++nq)
                        sc[nq][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), qf[nq][s], sc[nq][kb], 0, 0, 0);
                }
            // ---- softmax per row block
            u32x4 pw[NQ][NPS];
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq) {
                const int i = iw0 + 32 * nq + n32;
                float mx = kNegBig;
                if constexpr (FULL) {
#pragma unroll
                    for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sc[nq][kb][r]);
                } else {
#pragma unroll
                    for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int j = j0 + 32 * kb + 8 * (r >> 2) + 4 * jj + (r & 3);
                            // branch-free predicate (bitwise on purpose: no short-circuit control flow)
                            const bool okD = (j >= S) & (j <= i - W);
                            const bool okP = (j <= i) & ((!has_shared) | (j < S) | (j > i - W));
                            const bool ok = phaseD ? okD : okP;
                            sc[nq][kb][r] = ok ? sc[nq][kb][r] : kNegBig;
                            mx = fmaxf(mx, sc[nq][kb][r]);
                        }
                }
                mx = pair_max(mx) * p.scale_log2e; // scale > 0: max and scaling commute
                if (mx > m_ref[nq] + kLazy) {      // (masked rows have mx = -inf-like and never trigger)
                    const float m_new = mx;
                    const float alpha = __builtin_amdgcn_exp2f(m_ref[nq] - m_new);
                    l_run[nq] *= alpha;
#pragma unroll
                    for (int db = 0; db < NDB; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r) oacc[nq][db][r] *= alpha;
                    m_ref[nq] = m_new;
                }
                const float mr = m_ref[nq];
                float ps = 0.f;
#pragma unroll
                for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        float e = __builtin_amdgcn_exp2f(fmaf(sc[nq][kb][r], p.scale_log2e, -mr)); // raw v_exp_f32: tiny results flush to 0
                        if constexpr (!FULL) e = sc[nq][kb][r] <= kNegBig ? 0.f : e;
                        sc[nq][kb][r] = e;
                        ps += e;
                    }
                l_run[nq] += ps;
#pragma unroll
                for (int ks = 0; ks < NPS; ++ks) {
                    const int kb = ks >> 1, u = ks & 1;
                    pw[nq][ks].x = pack_bf16(sc[nq][kb][8 * u + 0], sc[nq][kb][8 * u + 1]);
                    pw[nq][ks].y = pack_bf16(sc[nq][kb][8 * u + 2], sc[nq][kb][8 * u + 3]);
                    pw[nq][ks].z = pack_bf16(sc[nq][kb][8 * u + 4], sc[nq][kb][8 * u + 5]);
                    pw[nq][ks].w = pack_bf16(sc[nq][kb][8 * u + 6], sc[nq][kb][8 * u + 7]);
                }
            }
            // ---- O^T += V^T P
#pragma unroll
            for (int ks = 0; ks < NPS; ++ks)
#pragma unroll
                for (int db = 0; db < NDB; ++db) {
                    const u32x4 a = *(const u32x4 *)(lbuf + KBUF + (db * NPS + ks) * VSTRIDE + vroff[db & 1]);
#pragma unroll
                    for (int nq = 0; nq < NQ; ++nq)
                        oacc[nq][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), as_bf16x8(pw[nq][ks]), oacc[nq][db], 0, 0, 0);
                }
        };
        if (any && iw0 <= iw_last) {
            if (full) tile_body(std::true_type{});
            else tile_body(std::false_type{});
        }
        // tile t+1 (loaded one iteration ago) goes to the other buffer; the loads of tile t+2 leave
        // before the barrier so that the wait at the barrier already overlaps their latency
        if (t + 1 < T) store_tile(buf ^ 1);
        if (t + 2 < T) load_tile(t + 2);
        __syncthreads();
    }

    // ---- normalise and store: lane (row n32, jj) holds dims 32db + 8a + 4jj + {0..3}
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const int i = iw0 + 32 * nq + n32;
        const float l = pair_sum(l_run[nq]);
        if (i >= p.n) continue;
        const float inv = 1.f / l;
        pod_bf16 *orow = p.out + ((size_t)i * p.Hq + head) * D;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                u32x2 o;
                o.x = pack_bf16(oacc[nq][db][4 * a + 0] * inv, oacc[nq][db][4 * a + 1] * inv);
                o.y = pack_bf16(oacc[nq][db][4 * a + 2] * inv, oacc[nq][db][4 * a + 3] * inv);
                *(u32x2 *)(orow + 32 * db + 8 * a + 4 * jj) = o;
            }
    }
}

} // namespace

int pod_launch_prefill(const pod_layout &ly, int layer, int n, const void *q, const void *k, const void *v,
                       const void *q_shared, const void *k_shared, float scale, void *out, hipStream_t st)
{
    (void)layer;
    prefill_params p;
    p.n = n; p.Hq = ly.Hq; p.Hkv = ly.Hkv; p.rep = ly.rep; p.S = ly.S; p.W = ly.W;
    p.q = (const pod_bf16 *)q; p.k = (const pod_bf16 *)k; p.v = (const pod_bf16 *)v;
    p.qs = (const pod_bf16 *)q_shared; p.ks = (const pod_bf16 *)k_shared;
    p.out = (pod_bf16 *)out;
    p.scale_log2e = scale * 1.4426950408889634f;
    if (scale <= 0.f) return pod_fail(POD_ERR_INVALID_ARG, "scale must be positive");
    constexpr int NQ = 1;
    const int BM = 128 * NQ;
    const dim3 grid((unsigned)((n + BM - 1) / BM) * (unsigned)ly.Hq);
    // dynamic LDS: 2 buffers x (key fragments + V^T fragments), see the kernel
    const auto lds_bytes = [](int D) { return 2 * ((kBN / 32) * (D / 16) + (D / 32) * (kBN / 16)) * 1024; };
    static bool attr_done = false; // raising the limit past 64 KB is needed once per process
    if (!attr_done) {
        POD_HIP_TRY(hipFuncSetAttribute((const void *)prefill_kernel<128, NQ>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(128)));
        POD_HIP_TRY(hipFuncSetAttribute((const void *)prefill_kernel<64, NQ>, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(64)));
        attr_done = true;
    }
    if (ly.D == 128)
        hipLaunchKernelGGL((prefill_kernel<128, NQ>), grid, dim3(256), lds_bytes(128), st, p);
    else
        hipLaunchKernelGGL((prefill_kernel<64, NQ>), grid, dim3(256), lds_bytes(64), st, p);
    POD_HIP_TRY(hipGetLastError());
    return POD_OK;
}
