// Measurement aids (not part of the method): kernels of known work that calibrate the roofs the similarity
// kernels are held against.  See "Measurement and test aids" in include/krul.h.
//
//  * calibration_block_kernel: the inner step of the similarity kernels with no memory traffic -- per 32-key x
//    32-row block of logits a chain of 8 MFMAs (32x32x16, bf16) and/or the vector work of its 16 logits per
//    lane (scale-and-shift, exp2, sum of squares, cross term, binary16 copy) and/or the 8 operand reads from
//    LDS.  Its times are the floors "matrix cores alone", "vector units alone", "both in one wave".
#include "krul_mfma_kernel.h"

namespace krul {
namespace {

typedef _Float16 cal_h2 __attribute__((ext_vector_type(2)));
typedef float cal_f2 __attribute__((ext_vector_type(2)));

// FL bits: 1 MFMA chains, 2 vector work, 4 operand reads from LDS.  RB: 32-row blocks of logits per block of
// keys (1 or 2: the two forms of the similarity kernels).  One workgroup of 8 waves per CU (2 waves per SIMD).
template <int RB, int FL>
__global__ __launch_bounds__(512, 2) void calibration_block_kernel(float *out, int iters, float seed)
{
    __shared__ __attribute__((aligned(16384))) unsigned char lds[65536];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < 65536 / 4; i += blockDim.x) reinterpret_cast<float *>(lds)[i] = seed * (i & 1023) * 1e-3f;
    __syncthreads();
    bf16x8 qf[RB][8], aop[8];
    for (int r = 0; r < RB; ++r)
        for (int ks = 0; ks < 8; ++ks)
            for (int i = 0; i < 8; ++i) qf[r][ks][i] = (__bf16)(seed * 0.01f * (i + ks + r));
    for (int ks = 0; ks < 8; ++ks) aop[ks] = qf[0][(ks + 3) & 7];
    f32x16 acc[RB];
    cal_h2 e2[RB][2][8];
    for (int r = 0; r < RB; ++r) {
        // (no two of these values are equal or a fixed distance apart, so that no exponential below can serve twice)
        for (int v = 0; v < 16; ++v) acc[r][v] = seed * 0.001f * (float)((v * v + 3 * v + 1) * (r + 1)) + 1e-4f * lane;
        for (int b = 0; b < 2; ++b)
            for (int i = 0; i < 8; ++i) e2[r][b][i] = cal_h2{(_Float16)(seed * 0.1f), (_Float16)(seed * 0.2f)};
    }
    float tn[RB], td[RB];
    for (int r = 0; r < RB; ++r) tn[r] = td[r] = 0.f;
    const float cs = 0.127f;
    const int a_base = (lane & 31) * 256 + (((lane >> 5) ^ (lane & 15)) << 4) + (wave & 1) * 8192;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            // (moves every turn and with b: nothing of the vector work is loop-invariant or shared between blocks)
            const float negm = -seed * 0.01f - (float)(2 * it + b) * 1.3e-6f;
            if (!(FL & 4)) asm volatile("" : "+v"(aop[0]));   // (opaque: no chain is the same as last turn's)
            if (FL & 4) {
                const unsigned char *slot = lds + ((it * 2 + b) & 3) * 16384;
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) aop[ks] = *reinterpret_cast<const bf16x8 *>(slot + (a_base ^ (ks << 5)));
            }
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                // the vector work of the block formed one turn ago (in acc[r]) beside the chain that forms the next
                f32x16 x = acc[r];
                if (FL & 2) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) x[v] = fmaf(x[v], cs, negm);
                }
                f32x16 nx;
#pragma unroll
                for (int v = 0; v < 16; ++v) nx[v] = 0.f;
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    if (FL & 1) {
                        nx = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[ks], qf[r][ks], nx, 0, 0, 0);
                        asm volatile("" : "+v"(nx));
                    }
                    if (FL & 2) {
                        const float ea = __builtin_amdgcn_exp2f(x[2 * ks]), eb = __builtin_amdgcn_exp2f(x[2 * ks + 1]);
                        tn[r] = fmaf(ea, ea, tn[r]);
                        tn[r] = fmaf(eb, eb, tn[r]);
                        td[r] = fmaf(ea, (float)e2[r][b][ks].x, td[r]);
                        td[r] = fmaf(eb, (float)e2[r][b][ks].y, td[r]);
                        e2[r][b][ks] = __builtin_convertvector((cal_f2{ea, eb}), cal_h2);
                        asm volatile("" : "+v"(tn[r]), "+v"(td[r]));
                    }
                }
                if (FL & 1) acc[r] = nx;
                else if (FL & 4) acc[r][0] += (float)aop[b][0];
            }
        }
    }
    float s = 0.f;
    for (int r = 0; r < RB; ++r) {
        s += tn[r] + td[r];
        for (int v = 0; v < 16; ++v) s += acc[r][v];
        for (int b = 0; b < 2; ++b)
            for (int i = 0; i < 8; ++i) s += (float)e2[r][b][i].x;
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <int RB>
hipError_t launch_block(int flags, float *out, int iters, hipStream_t st)
{
    const dim3 grid(256), block(512);
    switch (flags & 7) {
    case 1: hipLaunchKernelGGL((calibration_block_kernel<RB, 1>), grid, block, 0, st, out, iters, 1.0f); break;
    case 2: hipLaunchKernelGGL((calibration_block_kernel<RB, 2>), grid, block, 0, st, out, iters, 1.0f); break;
    case 3: hipLaunchKernelGGL((calibration_block_kernel<RB, 3>), grid, block, 0, st, out, iters, 1.0f); break;
    case 5: hipLaunchKernelGGL((calibration_block_kernel<RB, 5>), grid, block, 0, st, out, iters, 1.0f); break;
    case 7: hipLaunchKernelGGL((calibration_block_kernel<RB, 7>), grid, block, 0, st, out, iters, 1.0f); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace
}  // namespace krul

using namespace krul;

extern "C" int krul_calibration_block(int32_t row_blocks, int32_t parts, int32_t iters, float *out, void *stream)
{
    if (!out || iters <= 0 || ((uintptr_t)out & 3)) return KRUL_EINVAL;
    hipError_t e;
    if (row_blocks == 1) e = launch_block<1>(parts, out, iters, static_cast<hipStream_t>(stream));
    else if (row_blocks == 2) e = launch_block<2>(parts, out, iters, static_cast<hipStream_t>(stream));
    else return KRUL_EINVAL;
    if (e == hipErrorInvalidValue) return KRUL_EINVAL;
    return e == hipSuccess ? KRUL_OK : KRUL_ELAUNCH;
}
