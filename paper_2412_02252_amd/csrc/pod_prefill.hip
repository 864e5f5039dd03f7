// Prefill attention for PoD: causal flash attention on bf16 MFMA with two logit sources.
//
// For query i and key j <= i (Eq. 3 of the paper with the window taken at the query's own
// position): j is proximal if j < S or j > i - W and its logit is q_l[i].k_l[j]; otherwise it is
// distant and its logit is the block's lowest layer's, q_a[i].k_a[j].  One softmax over all
// j <= i (Eq. 4 / appendix), values always v_l.  A key tile is "own" (all proximal), "shared"
// (all distant) or mixed; mixed tiles compute both products and select per element.
//
// Tiling: a workgroup of 4 waves takes BM = 128*NQ query rows of one head; each wave owns
// 32*NQ rows and keeps Q (and the shared Q) as MFMA B operands in registers for the whole
// key loop.  Key/value tiles of BN = 64 tokens go through LDS, written in MFMA A-operand
// *fragment order* (64 lanes x 16 bytes per fragment) so that every read is one conflict-free
// ds_read_b128:
//   S^T[key][row] = K[key][:] . Q[row][:]     v_mfma_f32_32x32x16_bf16, A = K frag, B = Q
//   O^T[dim][row] = sum_key V[key][dim] P[key][row]               A = V^T frag, B = P
// Query row = MFMA column (lane % 32) in both, so softmax state, P and the output slice of a
// row stay in the same lane, and the S^T accumulators become the P operand without moving
// (the 8 keys a lane holds for one PV k-step are the keys of its 8 consecutive accumulators;
// V^T fragments are built for that key order).  V is transposed on the way into LDS: a thread
// loads the same 16-byte dim piece of 4 tokens and transposes the 4x8 block with v_perm_b32.
#include "pod_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kBN = 64;
constexpr float kNegBig = -1.0e30f;

struct prefill_params {
    int n, Hq, Hkv, rep, S, W;
    const pod_bf16 *q, *k, *v, *qs, *ks; // qs/ks NULL: own q,k serve every key
    pod_bf16 *out;
    float scale_log2e;
};

__device__ inline bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ inline unsigned pack_bf16(float lo, float hi)
{
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    bf16x2 t = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(unsigned, t);
}

__device__ inline unsigned dword_of(const uint4 &u, int w) { return w == 0 ? u.x : w == 1 ? u.y : w == 2 ? u.z : u.w; }

template <int D, int NQ>
__global__ __launch_bounds__(256) void prefill_kernel(prefill_params p)
{
    constexpr int CPR = D / 8;       // 16-byte pieces per row
    constexpr int KST = D / 16;      // QK k-steps (32x32x16)
    constexpr int NDB = D / 32;      // output dim blocks
    constexpr int NKB = kBN / 32;    // key blocks per tile
    constexpr int NPS = kBN / 16;    // PV k-steps per tile
    constexpr int BM = 128 * NQ;

    __shared__ uint4 ldsK[NKB * KST * 64];  // own-key fragments   [kb][s][64 lanes]
    __shared__ uint4 ldsKs[NKB * KST * 64]; // shared-key fragments
    __shared__ uint4 ldsV[NDB * NPS * 64];  // V^T fragments       [db][ks][64 lanes]

    const int nqt = (p.n + BM - 1) / BM;
    const int qt = nqt - 1 - blockIdx.x; // heaviest tiles first
    const int head = blockIdx.y, kvh = head / p.rep;
    const int i0 = qt * BM;
    const int i_last = min(i0 + BM, p.n) - 1;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n32 = lane & 31, jj = lane >> 5;
    const int iw0 = i0 + wave * 32 * NQ;           // first row of this wave
    const int iw_last = min(iw0 + 32 * NQ, p.n) - 1; // may be < iw0: the wave has no rows
    const bool has_shared = p.qs != nullptr;

    // Q (and shared Q) as B operands: lane (row n32, jj) holds dims 16s + 8jj .. +7
    bf16x8 qf[NQ][KST], qsf[NQ][KST];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const int row = min(iw0 + 32 * nq + n32, p.n - 1);
        const uint4 *qr = (const uint4 *)(p.q + ((size_t)row * p.Hq + head) * D);
        const uint4 *qsr = (const uint4 *)((has_shared ? p.qs : p.q) + ((size_t)row * p.Hq + head) * D);
#pragma unroll
        for (int s = 0; s < KST; ++s) {
            qf[nq][s] = as_bf16x8(qr[2 * s + jj]);
            qsf[nq][s] = as_bf16x8(qsr[2 * s + jj]);
        }
    }

    f32x16 oacc[NQ][NDB];
    float m_run[NQ], l_run[NQ];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        m_run[nq] = kNegBig; l_run[nq] = 0.f;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[nq][db][r] = 0.f;
    }

    const int ntiles = i_last / kBN + 1;
    for (int kt = 0; kt < ntiles; ++kt) {
        const int j0 = kt * kBN, j1 = j0 + kBN - 1;
        // what this workgroup's rows need from the tile
        bool need_own = true, need_sh = false;
        if (has_shared) {
            const bool all_prox = (j1 < p.S) || (j0 > i_last - p.W);
            const bool all_dist = (j0 >= p.S) && (j1 <= i0 - p.W);
            need_own = !all_dist; need_sh = !all_prox;
        }
        __syncthreads(); // previous tile's fragments are no longer read
        // ---- K tiles -> fragment order.  Thread: piece c of row r0 + (256/CPR)*it
        {
            const int c = tid % CPR, r0 = tid / CPR;
#pragma unroll
            for (int it = 0; it < kBN * CPR / 256; ++it) {
                const int r = r0 + (256 / CPR) * it; // key within the tile
                const int key = min(j0 + r, p.n - 1);
                const size_t g = ((size_t)key * p.Hkv + kvh) * CPR + c;
                const int s = c >> 1, cj = c & 1;
                const int slot = ((r & 31) + 32 * cj) ^ ((s & 3) | (cj << 2));
                const int f = ((r >> 5) * KST + s) * 64 + slot;
                if (need_own) ldsK[f] = ((const uint4 *)p.k)[g];
                if (need_sh) ldsKs[f] = ((const uint4 *)p.ks)[g];
            }
        }
        // ---- V tile -> V^T fragments.  Thread: piece c, 4 tokens 16*ku + 8*half + 4*vj + {0..3}
        {
            const int c = tid % CPR, rest = tid / CPR;
            if (rest < 16) {
                const int half = rest & 1, vj = (rest >> 1) & 1, ku = rest >> 2;
                uint4 t[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int key = min(j0 + 16 * ku + 8 * half + 4 * vj + e, p.n - 1);
                    t[e] = ((const uint4 *)p.v)[((size_t)key * p.Hkv + kvh) * CPR + c];
                }
#pragma unroll
                for (int dlt = 0; dlt < 8; ++dlt) {
                    const unsigned sel = (dlt & 1) ? 0x07060302u : 0x05040100u;
                    uint2 pk;
                    pk.x = __builtin_amdgcn_perm(dword_of(t[1], dlt >> 1), dword_of(t[0], dlt >> 1), sel);
                    pk.y = __builtin_amdgcn_perm(dword_of(t[3], dlt >> 1), dword_of(t[2], dlt >> 1), sel);
                    const int dim = 8 * c + dlt, db = dim >> 5;
                    const int l = (dim & 31) + 32 * vj;
                    const int slot = l ^ (((l >> 3) & 3) | (((l >> 5) ^ (db & 1)) << 2));
                    uint2 *dst = (uint2 *)&ldsV[(db * NPS + ku) * 64 + slot];
                    dst[half] = pk;
                }
            }
        }
        __syncthreads();

        if (j0 > iw_last) continue; // tile lies above this wave's diagonal (wave-uniform)
        // wave-level needs
        bool own_w = true, sh_w = false;
        if (has_shared) {
            const bool all_prox = (j1 < p.S) || (j0 > iw_last - p.W);
            const bool all_dist = (j0 >= p.S) && (j1 <= iw0 - p.W);
            own_w = !all_dist; sh_w = !all_prox;
        }
        const bool diag = j1 > iw0; // some (row, key) pair of this wave is not visible

#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
            f32x16 sc[NKB];
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) {
                f32x16 so, ss;
#pragma unroll
                for (int r = 0; r < 16; ++r) { so[r] = 0.f; ss[r] = 0.f; }
                if (own_w) {
#pragma unroll
                    for (int s = 0; s < KST; ++s) {
                        const uint4 a = ldsK[(kb * KST + s) * 64 + (lane ^ ((s & 3) | (jj << 2)))];
                        so = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), qf[nq][s], so, 0, 0, 0);
                    }
                }
                if (sh_w) {
#pragma unroll
                    for (int s = 0; s < KST; ++s) {
                        const uint4 a = ldsKs[(kb * KST + s) * 64 + (lane ^ ((s & 3) | (jj << 2)))];
                        ss = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), qsf[nq][s], ss, 0, 0, 0);
                    }
                }
                const int i = iw0 + 32 * nq + n32;
                if (own_w && sh_w) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int j = j0 + 32 * kb + 8 * (r >> 2) + 4 * jj + (r & 3);
                        const bool prox = (j < p.S) || (j > i - p.W);
                        sc[kb][r] = prox ? so[r] : ss[r];
                    }
                } else {
                    sc[kb] = own_w ? so : ss;
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) sc[kb][r] *= p.scale_log2e;
                if (diag) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int j = j0 + 32 * kb + 8 * (r >> 2) + 4 * jj + (r & 3);
                        if (j > i) sc[kb][r] = kNegBig;
                    }
                }
            }
            // online softmax for row n32 (this lane holds half of the tile's keys)
            float mx = kNegBig;
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sc[kb][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run[nq], mx);
            const float alpha = exp2f(m_run[nq] - m_new);
            float ps = 0.f;
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    // a fully masked row keeps m = kNegBig: exp2(0) would count masked keys
                    const float e = sc[kb][r] <= kNegBig ? 0.f : exp2f(sc[kb][r] - m_new);
                    sc[kb][r] = e;
                    ps += e;
                }
            ps += __shfl_xor(ps, 32);
            l_run[nq] = l_run[nq] * alpha + ps;
            m_run[nq] = m_new;
#pragma unroll
            for (int db = 0; db < NDB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[nq][db][r] *= alpha;
            // O^T += V^T P
#pragma unroll
            for (int ks = 0; ks < NPS; ++ks) {
                const int kb = ks >> 1, u = ks & 1;
                uint4 pw;
                pw.x = pack_bf16(sc[kb][8 * u + 0], sc[kb][8 * u + 1]);
                pw.y = pack_bf16(sc[kb][8 * u + 2], sc[kb][8 * u + 3]);
                pw.z = pack_bf16(sc[kb][8 * u + 4], sc[kb][8 * u + 5]);
                pw.w = pack_bf16(sc[kb][8 * u + 6], sc[kb][8 * u + 7]);
#pragma unroll
                for (int db = 0; db < NDB; ++db) {
                    const int slot = lane ^ (((lane >> 3) & 3) | (((lane >> 5) ^ (db & 1)) << 2));
                    const uint4 a = ldsV[(db * NPS + ks) * 64 + slot];
                    oacc[nq][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), as_bf16x8(pw), oacc[nq][db], 0, 0, 0);
                }
            }
        }
    }

    // ---- normalise and store: lane (row n32, jj) holds dims 32db + 8a + 4jj + {0..3}
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
        const int i = iw0 + 32 * nq + n32;
        if (i >= p.n) continue;
        const float inv = 1.f / l_run[nq];
        pod_bf16 *orow = p.out + ((size_t)i * p.Hq + head) * D;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                uint2 o;
                o.x = pack_bf16(oacc[nq][db][4 * a + 0] * inv, oacc[nq][db][4 * a + 1] * inv);
                o.y = pack_bf16(oacc[nq][db][4 * a + 2] * inv, oacc[nq][db][4 * a + 3] * inv);
                *(uint2 *)(orow + 32 * db + 8 * a + 4 * jj) = o;
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
    constexpr int NQ = 1;
    const int BM = 128 * NQ;
    const dim3 grid((unsigned)((n + BM - 1) / BM), (unsigned)ly.Hq);
    if (ly.D == 128)
        hipLaunchKernelGGL((prefill_kernel<128, NQ>), grid, dim3(256), 0, st, p);
    else
        hipLaunchKernelGGL((prefill_kernel<64, NQ>), grid, dim3(256), 0, st, p);
    POD_HIP_TRY(hipGetLastError());
    return POD_OK;
}
