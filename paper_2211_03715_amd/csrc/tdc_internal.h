// Internal declarations shared by the translation units of libtdc.so (not installed).
//
// Weight re-layout ("packed", frag-major) used by every MFMA kernel.  A weight matrix
// Wt[k][m] (k = contraction index, m = output channel) is padded with zeros to
// multiples of 16 in both directions and stored as
//     Wp[mb][kg][lane][j],   mb = m/16, kg = k/16, lane = 0..63, j = 0..3
//     Wp[mb][kg][lane][j] = Wt[16*kg + 4*(lane/16) + j][16*mb + lane%16]
// so that one 16-byte load per lane yields the A operands of four consecutive
// v_mfma_f32_16x16x4_f32 steps (A[m = lane%16][k = lane/16]) and a wavefront's load is
// one contiguous 1 KiB run.  The matching B operand of step j is
// B[k = 16*kg + 4*(lane/16) + j][p = lane%16]  (see tdc_mfma.h for why this order).
//   stage 1 (Eq. 2): k = c,                      m = d1   -> Uin_p  [NB1][KG1]
//   stage 2 (Eq. 3): k = (r*K + s)*R1P + d1,     m = d2   -> core_p [NB2][K*K*NB1]
//   stage 3 (Eq. 4): k = d2,                     m = n    -> Uout_p [NB3][NB2]
// with R1P = 16*NB1 >= R1, R2P = 16*NB2 >= R2, NP = 16*NB3 >= N, KG1 = ceil(C/16).
// Padded channels carry exact zeros through every stage, so the kernels need no
// remainder handling on the rank dimensions.
#ifndef TDC_INTERNAL_H
#define TDC_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tdc.h"
#include "tdc_measure.h"

// Optional output epilogue, applied as the last kernel stores y:
//   y = acc + bias[n] + residual[same element as y], then max(., 0) if relu.
struct TdcEpi {
    const float *bias;       // [N] or null
    const float *residual;   // shaped and laid out like y, or null
    int relu;
};

// Activation layouts the kernels read (GEMM kernels: template parameter ACT) and write.
enum { TDC_ACT_NCHW = 0, TDC_ACT_BLOCKED = 1, TDC_ACT_NHWC = 2 };

struct TdcDims {
    int B, C, N, H, W, R1, R2, K, stride, pad, Ho, Wo;
    int NB1, NB2, NB3;   // 16-blocks of the padded R1, R2, N
    int KG1;             // ceil(C/16)
    int nhwc;            // activations x, y (and an epilogue's residual) are [B][H][W][channels]; C % 4 == N % 4 == 0
    int s1_runs;         // NCHW one-launch kernels read x in 16-byte runs of four pixels (W % 4 == 0, x 16-byte
                         // aligned); U_in is then re-laid-out with k order 4*j + lane/16 instead of 4*(lane/16) + j
};

// Raises the dynamic-LDS limit of kernel `fn` to at least `bytes` on the current device.  The HIP
// attribute call is made once per kernel, device and size (a table remembers what was granted),
// so a launch path may call this every time; nothing is done for sizes the default limit covers.
hipError_t tdc_allow_lds(const void *fn, size_t bytes);

// ---- weight re-layout (tdc_pack.hip)
hipError_t tdc_launch_pack(const TdcDims &d, hipStream_t s, const float *U_in, const float *core,
                           const float *U_out, float *uin_p, float *core_p, float *uout_p);
hipError_t tdc_launch_pack_core(const TdcDims &d, hipStream_t s, const float *core, float *core_p);
// U_in as usual; Wm[R1][N][K][K] = core x_2 U_out into `wm`, then re-laid out into `wm_p` [NB3][K*K*NB1]
hipError_t tdc_launch_pack_merged(const TdcDims &d, hipStream_t s, const float *U_in, const float *core,
                                  const float *U_out, float *uin_p, float *wm, float *wm_p);
size_t tdc_packed_floats_uin(const TdcDims &d);
size_t tdc_packed_floats_core(const TdcDims &d);
size_t tdc_packed_floats_uout(const TdcDims &d);

// ---- plain kernels (tdc_naive.hip): raw weights, z1 [B][R1][H*W], z2 [B][R2][Ho*Wo]
hipError_t tdc_launch_naive(const TdcDims &d, hipStream_t s, const float *x, const float *U_in,
                            const float *core, const float *U_out, float *z1, float *z2, float *y, const TdcEpi &epi);

// ---- three MFMA GEMM kernels (tdc_gemm.hip): packed weights, z1 [B][R1P][H*W], z2 [B][R2P][Ho*Wo]
bool tdc_gemm_unit_supported(int mb, int pb);
hipError_t tdc_launch_split(const TdcDims &d, const tdc_tuning &t, hipStream_t s, const float *x,
                            const float *uin_p, const float *core_p, const float *uout_p,
                            float *z1, float *z2, float *y, const TdcEpi &epi);

// the dense K x K layer through the stage-2 kernel; `d` has R1 = C, R2 = N
hipError_t tdc_launch_dense(const TdcDims &d, const tdc_tuning &t, hipStream_t s, const float *x,
                            const float *w_p, float *y, const TdcEpi &epi);

// stage 1, then stages 2 and 3 as one implicit GEMM with the merged kernel
hipError_t tdc_launch_merged(const TdcDims &d, const tdc_tuning &t, hipStream_t s, const float *x,
                             const float *uin_p, const float *wm_p, float *z1, float *y, const TdcEpi &epi);

// MERGED in one launch (tdc_gemm.hip): `z1c` holds 8 copies of z1, `arrive` 8 x 32 words that start at zero,
// `status` is host-visible.  The grid (a multiple of 8, at most 256 workgroups of 512 threads) must be resident at once.
bool tdc_merged_xcd_supported(const tdc_tuning &t);
int tdc_merged_xcd_grid(const TdcDims &d, const tdc_tuning &t);
hipError_t tdc_launch_merged_xcd(const TdcDims &d, const tdc_tuning &t, hipStream_t s, const float *x, const float *uin_p,
                                 const float *wm_p, float *z1c, unsigned *arrive, unsigned *status, unsigned wait_limit,
                                 float *y, const TdcEpi &epi);
hipError_t tdc_merged_xcd_resident(int grid, bool nhwc, bool *fits);

// The one-launch kernels' launchers take `prepare_only`: do what must precede a first launch (raise the
// kernel's LDS limit) and return without launching, so that plan creation can get it out of the way
// of a later stream capture.
// ---- fused MFMA kernel (tdc_fused.hip)
struct TdcFusedGeom {
    int TH, TW;          // output tile
    int QH, QW, Q;       // input (halo'd) tile: QH = (TH-1)*stride + K, Q = QH*QW
    int QB, PBk;         // 16-pixel blocks of the input tile / output tile
    int tiles_x, tiles_y;
    int pitch1, pitch2;  // LDS row pitches (floats) of the z1 and z2 tiles
    bool weights_in_lds; // core and U_out are copied into LDS by every workgroup
    bool weights_fit;    // ... or would fit there (CHAIN streams them all the same when a wavefront uses them once)
    size_t lds_bytes;
};
bool tdc_fused_unit_supported(int mb1, int mb2, int mb3, int pb);
TdcFusedGeom tdc_fused_geometry(const TdcDims &d, int tile_h, int tile_w, int lds_limit);
hipError_t tdc_launch_fused(const TdcDims &d, const tdc_tuning &t, const TdcFusedGeom &g, hipStream_t s,
                            const float *x, const float *uin_p, const float *core_p,
                            const float *uout_p, float *y, const TdcEpi &epi, bool prepare_only = false);

// ---- fused MFMA kernel with stages 2 and 3 chained in registers (tdc_chain.hip, kernel in tdc_chain_kernel.h)
bool tdc_chain_supported(int nb2, int mb1, int pb);
TdcFusedGeom tdc_chain_geometry(const TdcDims &d, int tile_h, int tile_w, int nw, int pb, int lds_limit);
hipError_t tdc_launch_chain(const TdcDims &d, const tdc_tuning &t, const TdcFusedGeom &g, hipStream_t s,
                            const float *x, const float *uin_p, const float *core_p,
                            const float *uout_p, float *y, const TdcEpi &epi, bool prepare_only = false);

// ---- one-launch kernel: stage 1 into LDS, then the merged stage-2/3 convolution (tdc_fm.hip).
// Tuning fields: tile_h, tile_w, waves[0], mb[0] = stage-1 register tile, mb[1] = output-channel
// blocks per workgroup (the wavefronts split the contraction waves[0] / mb[1] ways).
bool tdc_fm_supported(const TdcDims &d, int tile_h, int tile_w, int nw, int mb1, int nbg);
TdcFusedGeom tdc_fm_geometry(const TdcDims &d, int tile_h, int tile_w, int nw, int nbg);
hipError_t tdc_launch_fm(const TdcDims &d, const tdc_tuning &t, const TdcFusedGeom &g, hipStream_t s, const float *x,
                         const float *uin_p, const float *wm_p, float *y, const TdcEpi &epi, bool prepare_only = false);

// Run-major stage 1 of the NCHW one-launch kernels (a lane loads four consecutive pixels of a row, aligned
// to 4 in image coordinates, with one 16-byte load).  FUSED and CHAIN plans use it in the throughput
// regime where the rows allow it (not in the latency regime: a run-major unit is 64 pixels, and the small
// tiles chosen there would mostly pad it -- measured 0.4 to 2.6 us slower per batch-1 layer).
inline bool tdc_runs_apply(const TdcDims &d, int cus)
{
    return !d.nhwc && d.W % 4 == 0 && (long)d.B * d.Ho * d.Wo >= 16L * cus;
}
// Runs per tile row (the most any tile column needs) for output tiles TW wide.
inline int tdc_runs_per_row(int W, int Wo, int TW, int K, int stride, int pad)
{
    const int QW = (TW - 1) * stride + K;
    int rpr = 1;
    for (int j0 = 0; j0 < Wo; j0 += TW) {
        const int w0 = j0 * stride - pad, wa = w0 > 0 ? (w0 & ~3) : 0;
        const int end = w0 + QW < W ? w0 + QW : W;
        const int runs = (end - wa + 3) / 4;
        rpr = runs > rpr ? runs : rpr;
    }
    return rpr;
}

// ---- selector (tdc_select.cpp): fills every zero field of `t`
struct TdcDeviceInfo {
    int cus;             // compute units
    int lds_per_wg;      // bytes of LDS one workgroup may use
};
// `model_us`, when not null, receives the latency estimate of the chosen tuning (0 for NAIVE)
int tdc_select(const TdcDims &d, const TdcDeviceInfo &dev, tdc_tuning *t, double *model_us);
// the terms of the estimate of a fully specified tuning `t` (what tdc_model_terms hands out)
int tdc_select_terms(const TdcDims &d, const TdcDeviceInfo &dev, const tdc_tuning &t, double *terms, const char **names,
                     int max_terms, int *n_terms, const char **model);

#endif
