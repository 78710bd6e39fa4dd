// Plain fp32 kernels for the three stages (Eqs. 2, 3, 4): one thread per output pixel,
// OT output channels in registers, weights read through wave-uniform addresses.  This
// variant reads the caller's weight layouts directly and supports every valid shape; it is
// the in-library yardstick the MFMA variants are measured against, not the fast path.
#include "tdc_internal.h"
#include "tdc_mfma.h"

namespace {

constexpr int OT = 8;      // output channels per thread
constexpr int TPB = 256;   // threads per block

// out[b][m][p] = sum_k in[b][k][p] * Wt[k][m]      (1x1 convolution; Eq. 2 and Eq. 4)
// in_nhwc / out_nhwc: that tensor is [b][p][channel] instead of [b][channel][p]
__global__ __launch_bounds__(TPB) void naive_pointwise(const float *__restrict__ in, const float *__restrict__ Wt,
                                                       float *__restrict__ out, int Kc, int M, int P, TdcEpi epi,
                                                       int in_nhwc, int out_nhwc)
{
    const int p = blockIdx.x * TPB + threadIdx.x;
    const int m0 = blockIdx.y * OT;
    const int b = blockIdx.z;
    if (p >= P) return;
    const float *inb = in + (size_t)b * Kc * P + (in_nhwc ? (size_t)p * Kc : (size_t)p);
    const size_t in_cs = in_nhwc ? 1 : (size_t)P;
    float acc[OT];
#pragma unroll
    for (int j = 0; j < OT; ++j) acc[j] = 0.f;
    for (int k = 0; k < Kc; ++k) {
        const float v = inb[(size_t)k * in_cs];
#pragma unroll
        for (int j = 0; j < OT; ++j)
            if (m0 + j < M) acc[j] = fmaf(v, Wt[(size_t)k * M + m0 + j], acc[j]);
    }
#pragma unroll
    for (int j = 0; j < OT; ++j)
        if (m0 + j < M) {
            const size_t idx = out_nhwc ? ((size_t)b * P + p) * M + m0 + j : ((size_t)b * M + m0 + j) * P + p;
            out[idx] = tdc_apply_epilogue(epi, acc[j], m0 + j, idx);
        }
}

// z2[b][d2][i][j] = sum_{d1,r,s} z1pad[b][d1][i*st+r-pad][j*st+s-pad] * core[d1][d2][r][s]      (Eq. 3)
__global__ __launch_bounds__(TPB) void naive_core(TdcDims d, const float *__restrict__ z1,
                                                  const float *__restrict__ core, float *__restrict__ z2)
{
    const int P = d.Ho * d.Wo;
    const int p = blockIdx.x * TPB + threadIdx.x;
    const int m0 = blockIdx.y * OT;
    const int b = blockIdx.z;
    if (p >= P) return;
    const int i = p / d.Wo, j = p % d.Wo;
    const int h0 = i * d.stride - d.pad, w0 = j * d.stride - d.pad;
    const int HW = d.H * d.W;
    const float *zb = z1 + (size_t)b * d.R1 * HW;
    float acc[OT];
#pragma unroll
    for (int o = 0; o < OT; ++o) acc[o] = 0.f;
    for (int d1 = 0; d1 < d.R1; ++d1)
        for (int r = 0; r < d.K; ++r) {
            const int h = h0 + r;
            if (h < 0 || h >= d.H) continue;
            for (int s = 0; s < d.K; ++s) {
                const int w = w0 + s;
                if (w < 0 || w >= d.W) continue;
                const float v = zb[(size_t)d1 * HW + h * d.W + w];
#pragma unroll
                for (int o = 0; o < OT; ++o)
                    if (m0 + o < d.R2)
                        acc[o] = fmaf(v, core[(((size_t)d1 * d.R2 + m0 + o) * d.K + r) * d.K + s], acc[o]);
            }
        }
#pragma unroll
    for (int o = 0; o < OT; ++o)
        if (m0 + o < d.R2) z2[((size_t)b * d.R2 + m0 + o) * P + p] = acc[o];
}

}  // namespace

hipError_t tdc_launch_naive(const TdcDims &d, hipStream_t s, const float *x, const float *U_in,
                            const float *core, const float *U_out, float *z1, float *z2, float *y, const TdcEpi &epi)
{
    const int HW = d.H * d.W, P = d.Ho * d.Wo;
    hipLaunchKernelGGL(naive_pointwise, dim3((HW + TPB - 1) / TPB, (d.R1 + OT - 1) / OT, d.B), dim3(TPB), 0, s,
                       x, U_in, z1, d.C, d.R1, HW, TdcEpi{nullptr, nullptr, 0}, d.nhwc, 0);
    hipLaunchKernelGGL(naive_core, dim3((P + TPB - 1) / TPB, (d.R2 + OT - 1) / OT, d.B), dim3(TPB), 0, s,
                       d, z1, core, z2);
    hipLaunchKernelGGL(naive_pointwise, dim3((P + TPB - 1) / TPB, (d.N + OT - 1) / OT, d.B), dim3(TPB), 0, s,
                       z2, U_out, y, d.R2, d.N, P, epi, 0, d.nhwc);
    return hipGetLastError();
}
