// Device helpers around v_mfma_f32_16x16x4_f32 (gfx950), shared by the GEMM and fused kernels.
//
// Operand layout of one step D += A*B with A 16x4, B 4x16, D 16x16, 64 lanes:
//   A : lane l holds A[m = l%16][k = l/16]
//   B : lane l holds B[k = l/16][p = l%16]
//   D : lane l holds D[m = 4*(l/16) + i][p = l%16] in register i = 0..3
// Here m is an output channel, p a pixel and k the contraction index, so pixels run
// along the lanes: activation loads and stores are contiguous in NCHW.
#ifndef TDC_MFMA_H
#define TDC_MFMA_H

#include <hip/hip_runtime.h>

typedef float tdc_f4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ tdc_f4 tdc_mfma(float a, float b, tdc_f4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// Four A operands (k-steps 4*kg .. 4*kg+3 of 16-channel block mb) from a packed weight array.
__device__ __forceinline__ tdc_f4 tdc_load_a4(const float *__restrict__ wp, int mb, int kgroups, int kg, int lane)
{
    const tdc_f4 *p = reinterpret_cast<const tdc_f4 *>(wp);
    return p[((size_t)mb * kgroups + kg) * 64 + lane];
}

// acc[MB][PB] += A(mb, 4 steps) * B(pb, 4 steps); the step loop is outermost so that
// consecutive MFMAs write different accumulators.
template <int MB, int PB>
__device__ __forceinline__ void tdc_mma_group(tdc_f4 (&acc)[MB][PB], const tdc_f4 (&a)[MB], const float (&b)[PB][4],
                                              int mvalid)
{
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            if (mb < mvalid) {
#pragma unroll
                for (int pb = 0; pb < PB; ++pb) acc[mb][pb] = tdc_mfma(a[mb][j], b[pb][j], acc[mb][pb]);
            }
}

#endif
