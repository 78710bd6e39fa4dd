// Weight re-layout kernels: caller layouts -> the frag-major packed layout of tdc_internal.h.
// The paper (section 5.2) converts its core weights to a coalescing-friendly layout once,
// offline; this is the same step for this library's MFMA operand order.
#include "tdc_internal.h"

size_t tdc_packed_floats_uin(const TdcDims &d) { return (size_t)d.NB1 * d.KG1 * 256; }
size_t tdc_packed_floats_core(const TdcDims &d) { return (size_t)d.NB2 * d.K * d.K * d.NB1 * 256; }
size_t tdc_packed_floats_uout(const TdcDims &d) { return (size_t)d.NB3 * d.NB2 * 256; }

namespace {

// e = ((mb*KG + kg)*64 + lane)*4 + j  ->  k = 16*kg + 4*(lane/16) + j, m = 16*mb + lane%16
__device__ __forceinline__ void unpack_index(size_t e, int kgroups, int &mb, int &kg, int &k16, int &m)
{
    const int j = (int)(e & 3);
    const int lane = (int)((e >> 2) & 63);
    const size_t blk = e >> 8;
    kg = (int)(blk % kgroups);
    mb = (int)(blk / kgroups);
    k16 = 4 * (lane >> 4) + j;
    m = 16 * mb + (lane & 15);
}

__global__ void pack_uin_kernel(TdcDims d, const float *__restrict__ U_in, float *__restrict__ out, size_t total)
{
    size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= total) return;
    int mb, kg, k16, m;
    unpack_index(e, d.KG1, mb, kg, k16, m);
    if (d.s1_runs) k16 = 4 * (k16 & 3) + (k16 >> 2);      // component j of lane group g holds channel 4*j + g
    const int c = 16 * kg + k16;
    out[e] = (c < d.C && m < d.R1) ? U_in[(size_t)c * d.R1 + m] : 0.f;
}

__global__ void pack_core_kernel(TdcDims d, const float *__restrict__ core, float *__restrict__ out, size_t total)
{
    size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= total) return;
    int mb, kg, k16, m;
    unpack_index(e, d.K * d.K * d.NB1, mb, kg, k16, m);
    const int tap = kg / d.NB1;              // r*K + s
    const int d1 = 16 * (kg % d.NB1) + k16;
    const int r = tap / d.K, s = tap % d.K;
    out[e] = (d1 < d.R1 && m < d.R2) ? core[(((size_t)d1 * d.R2 + m) * d.K + r) * d.K + s] : 0.f;
}

__global__ void pack_uout_kernel(TdcDims d, const float *__restrict__ U_out, float *__restrict__ out, size_t total)
{
    size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= total) return;
    int mb, kg, k16, m;
    unpack_index(e, d.NB2, mb, kg, k16, m);
    const int d2 = 16 * kg + k16;
    out[e] = (d2 < d.R2 && m < d.N) ? U_out[(size_t)d2 * d.N + m] : 0.f;
}

// Wm[d1][n][r][s] = sum_d2 core[d1][d2][r][s] * U_out[d2][n]: stage 3 folded into the core.
__global__ void merge_core_uout_kernel(TdcDims d, const float *__restrict__ core, const float *__restrict__ U_out,
                                       float *__restrict__ wm, size_t total)
{
    size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= total) return;
    const int KK = d.K * d.K;
    const int tap = (int)(e % KK);
    const int n = (int)((e / KK) % d.N);
    const int d1 = (int)(e / ((size_t)KK * d.N));
    float acc = 0.f;
    for (int d2 = 0; d2 < d.R2; ++d2) acc += core[((size_t)d1 * d.R2 + d2) * KK + tap] * U_out[(size_t)d2 * d.N + n];
    wm[e] = acc;
}

}  // namespace

hipError_t tdc_launch_pack_merged(const TdcDims &d, hipStream_t s, const float *U_in, const float *core,
                                  const float *U_out, float *uin_p, float *wm, float *wm_p)
{
    const int T = 256;
    const size_t n1 = tdc_packed_floats_uin(d), nm = (size_t)d.R1 * d.N * d.K * d.K;
    hipLaunchKernelGGL(pack_uin_kernel, dim3((unsigned)((n1 + T - 1) / T)), dim3(T), 0, s, d, U_in, uin_p, n1);
    hipLaunchKernelGGL(merge_core_uout_kernel, dim3((unsigned)((nm + T - 1) / T)), dim3(T), 0, s, d, core, U_out, wm, nm);
    TdcDims m = d;          // the merged kernel is a core tensor with R2 = N
    m.R2 = d.N;
    m.NB2 = d.NB3;
    const size_t n2 = tdc_packed_floats_core(m);
    hipLaunchKernelGGL(pack_core_kernel, dim3((unsigned)((n2 + T - 1) / T)), dim3(T), 0, s, m, wm, wm_p, n2);
    return hipGetLastError();
}

hipError_t tdc_launch_pack(const TdcDims &d, hipStream_t s, const float *U_in, const float *core,
                           const float *U_out, float *uin_p, float *core_p, float *uout_p)
{
    const int T = 256;
    size_t n1 = tdc_packed_floats_uin(d), n2 = tdc_packed_floats_core(d), n3 = tdc_packed_floats_uout(d);
    hipLaunchKernelGGL(pack_uin_kernel, dim3((unsigned)((n1 + T - 1) / T)), dim3(T), 0, s, d, U_in, uin_p, n1);
    hipLaunchKernelGGL(pack_core_kernel, dim3((unsigned)((n2 + T - 1) / T)), dim3(T), 0, s, d, core, core_p, n2);
    hipLaunchKernelGGL(pack_uout_kernel, dim3((unsigned)((n3 + T - 1) / T)), dim3(T), 0, s, d, U_out, uout_p, n3);
    return hipGetLastError();
}

hipError_t tdc_launch_pack_core(const TdcDims &d, hipStream_t s, const float *core, float *core_p)
{
    const int T = 256;
    const size_t n2 = tdc_packed_floats_core(d);
    hipLaunchKernelGGL(pack_core_kernel, dim3((unsigned)((n2 + T - 1) / T)), dim3(T), 0, s, d, core, core_p, n2);
    return hipGetLastError();
}
