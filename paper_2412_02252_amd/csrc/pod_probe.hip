// Measurement aid for the prefill kernel's roofline: how busy can the matrix pipes of this chip be kept when every
// 32x32x16 bf16 MFMA takes one operand fragment (16 bytes per lane, 1 KB per wave) out of LDS, as a flash-attention
// kernel with 32 query rows per wave must (K as the A operand of S^T = K Q^T, V^T as the A operand of O^T = V^T P^T)?
//
// A CU's four SIMDs each retire one such MFMA per 32 cycles at best, i.e. they ask LDS for 4 KB per 32 cycles =
// 128 bytes per cycle, which is the LDS's whole bandwidth.  The loops below measure where that leaves the pipes:
// two waves per SIMD (the prefill kernel's occupancy), 8 fragments in a ring, the fragment for the MFMA two groups
// ahead requested while the current one runs.
//   variant 0: MFMAs only (operands stay in registers)             -> the pipe's own rate
//   variant 1: one LDS fragment per MFMA
//   variant 2: one LDS fragment per MFMA + 3 fma + 1 exp per MFMA   (about the prefill kernel's vector work per MFMA,
//              which is 4.75 vector instructions of which one exponential)
//   variant 3: one LDS fragment per TWO MFMAs + 3 fma + 1 exp per MFMA (what 64 query rows per wave would give; at
//              head dimension 128 that needs ~290 registers per wave and does not fit two waves per SIMD)
// The caller times the launch; MFMAs per SIMD = iters * 8 * (2 for variant 3, else 1) * 2 waves.
#include "pod_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

template <int FROM_LDS, int MPL, int KF, int KE>
__global__ __launch_bounds__(512) void mfma_feed_kernel(float *out, int iters)
{
    extern __shared__ u32x4 feed_lds[];   // 80 KB asked for at launch: one workgroup (8 waves) per CU
    for (int i = threadIdx.x; i < 4096; i += blockDim.x) feed_lds[i] = u32x4{0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u};
    __syncthreads();
    f32x16 acc[4];
    for (int a = 0; a < 4; ++a)
        for (int r = 0; r < 16; ++r) acc[a][r] = 0.f;
    bf16x8 bv, bv2;
    for (int i = 0; i < 8; ++i) { bv[i] = (__bf16)(0.5f); bv2[i] = (__bf16)(0.25f); }
    float x[16];
    for (int i = 0; i < 16; ++i) x[i] = threadIdx.x * 0.01f + i;
    const float ca = 0.999f, cb = 0.001f;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // 256-byte rows, 16-byte pieces XOR-permuted: the conflict-free layout of a K tile read as the MFMA's A operand
    const int n32 = lane & 31, jj = lane >> 5;
    const u32x4 *base = feed_lds + (n32 * 16 + (jj ^ (n32 & 15)));
    u32x4 fr[8];
    for (int i = 0; i < 8; ++i) fr[i] = base[(i * 512 + wave * 64) & 4095];
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (FROM_LDS) asm volatile("s_waitcnt lgkmcnt(1)" ::: "memory");   // the fragment asked for two groups ago
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[u & 3]) : "v"(fr[u]), "v"(bv));
            if (MPL == 2) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[(u + 2) & 3]) : "v"(fr[u]), "v"(bv2));
            if (FROM_LDS) {
                fr[(u + 2) & 7] = base[((it * 8 + u) * 512 + wave * 64) & 4080];
                asm volatile("" : "+v"(fr[(u + 2) & 7]));
            }
#pragma unroll
            for (int f = 0; f < KF * MPL; ++f) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[f & 7]) : "v"(ca), "v"(cb));
#pragma unroll
            for (int e = 0; e < KE * MPL; ++e) asm volatile("v_exp_f32 %0, %0" : "+v"(x[8 + (e & 7)]));
        }
    }
    float s = 0.f;
    for (int a = 0; a < 4; ++a)
        for (int r = 0; r < 16; ++r) s += acc[a][r];
    for (int i = 0; i < 16; ++i) s += x[i];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <int FROM_LDS, int MPL, int KF, int KE>
int launch_feed(float *out, int wgs, int iters, hipStream_t st)
{
    const int lds = 80 * 1024;
    POD_HIP_TRY(hipFuncSetAttribute((const void *)mfma_feed_kernel<FROM_LDS, MPL, KF, KE>, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    hipLaunchKernelGGL((mfma_feed_kernel<FROM_LDS, MPL, KF, KE>), dim3(wgs), dim3(512), lds, st, out, iters);
    POD_HIP_TRY(hipGetLastError());
    return POD_OK;
}

} // namespace

int pod_launch_mfma_feed(int variant, int iters, float *out, size_t out_bytes, hipStream_t st)
{
    int dev = 0, cus = 256;
    POD_HIP_TRY(hipGetDevice(&dev));
    POD_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    if (out_bytes < (size_t)cus * 512 * sizeof(float))
        return pod_fail(POD_ERR_CAPACITY, "out has %zu bytes, needs %zu", out_bytes, (size_t)cus * 512 * sizeof(float));
    switch (variant) {
    case 0: return launch_feed<0, 1, 0, 0>(out, cus, iters, st);
    case 1: return launch_feed<1, 1, 0, 0>(out, cus, iters, st);
    case 2: return launch_feed<1, 1, 3, 1>(out, cus, iters, st);
    case 3: return launch_feed<1, 2, 3, 1>(out, cus, iters, st);
    default: return pod_fail(POD_ERR_INVALID_ARG, "variant %d outside [0, 3]", variant);
    }
}
