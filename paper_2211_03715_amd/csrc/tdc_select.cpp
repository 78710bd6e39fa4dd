// Tile / launch-parameter selector (host only).
//
// The paper picks its (TH, TW, TC) tile with an analytical model (section 5.3-5.5): a
// compute-latency term from the number of thread-block waves, then the smallest memory
// volume among the best few percent, and reports it about 25% behind an exhaustive search.
// That model describes one-thread-per-output-channel blocks on an NVIDIA SM; this selector
// keeps the method -- enumerate every tiling, score it with a closed-form latency estimate, no
// search on the device -- with terms that describe this library's kernels on CDNA4.
//
// Per workgroup, every stage costs   rounds * (unit + kgroups * (kg + mfma * MB*PB*share))
// where rounds = register tiles ("units") per wavefront, kgroups = 16-wide contraction steps
// per tile, and share >= 1 is the number of wavefronts that time-share one of the CU's four
// MFMA pipes.  A workgroup round over the chip repeats ceil(WGs / (CUs * resident)) times and
// one dependent launch adds a constant.  The coefficients (microseconds) were fitted by
// non-negative least squares to exhaustive sweeps on MI355X, separately for the latency regime
// (batch 1: one-launch and GEMM kernels, ~2500-6600 tunings per model) and the throughput regime
// (eight batch-1 to batch-64 layers: fused and chain kernels in both activation layouts and both
// forms of stage 1, ~30000 tunings); median relative errors 5-12%.  Each term enumeration below
// says what its terms stand for; the coefficients live in tdc_select_coef.h.
#include <algorithm>
#include <climits>
#include <cmath>

#include "tdc_internal.h"
#include "tdc_select_coef.h"

namespace {


inline int cdiv(int a, int b) { return (a + b - 1) / b; }

constexpr int kWavesPerCu = 32;   // 8 per SIMD

// Workgroups of `nw` wavefronts one compute unit holds at a time: as many as LDS allows, and as the
// vector registers allow -- `wps` wavefronts per SIMD (512 registers per lane and SIMD, divided by what
// the kernel instance uses), four SIMDs.  The throughput kernels use 140-250 registers, so a compute unit
// holds 8 to 12 of their wavefronts, not the 32 the hardware has slots for; tunings timed with 8-wavefront
// workgroups show it: a second workgroup per compute unit waits for the first to finish.
inline int resident_wgs(const TdcDeviceInfo &dev, size_t lds_bytes, int nw, int wps)
{
    return std::max(1, std::min({(int)(dev.lds_per_wg / std::max<size_t>(lds_bytes, 1)), 4 * wps / nw, 8}));
}

// Every estimate below is a dot product  sum_i coef[i] * term[i]  of fitted coefficients (microseconds; the tables in
// tdc_select_coef.h, written by `python -m paper_2211_03715_amd.autotune --fit`) with terms that are computed from the
// shape and the tuning alone.  tdc_model_terms() hands the terms out, so the fit needs no second copy of the model.

// FUSED.  Terms, all per workgroup round over the chip except the first:
enum {
    F_LAUNCH, F_S1_UNIT, F_S1_KG, F_S1_MFMA,       // constant; stage 1 per register tile, per k-group, per MFMA quad x pipe share
    F_S1R_UNIT, F_S1R_KG, F_S1R_MFMA,              // the same for the run-major form of stage 1 (64-pixel units)
    F_S2_KG_LDS, F_S2_KG_GLB, F_S2_MFMA,           // stage 2 per k-group with weights in LDS / streamed, per MFMA quad
    F_S3_UNIT, F_S3_KG_LDS, F_S3_KG_GLB, F_S3_MFMA,
    F_W_KB,                                        // KiB of weights copied into LDS, per co-resident workgroup
    F_X_MB_NCHW, F_X_MB_NHWC, F_X_MB_RUNS,         // MB of x a CU pulls, by the way it is read
    F_Y_MB_NCHW, F_Y_MB_NHWC,                      // MB of y a CU pushes
    F_X_ROWS, F_Y_ROWS,                            // NCHW: thousands of row segments a CU reads (4-byte loads only) / writes
    F_TERMS
};
const char *const kFusedTermNames[F_TERMS] = {"launch", "s1_unit", "s1_kg", "s1_mfma", "s1r_unit", "s1r_kg", "s1r_mfma",
                                              "s2_kg_lds", "s2_kg_glb", "s2_mfma", "s3_unit", "s3_kg_lds", "s3_kg_glb", "s3_mfma",
                                              "w_kb", "x_mb_nchw", "x_mb_nhwc", "x_mb_runs", "y_mb_nchw", "y_mb_nhwc", "x_rows", "y_rows"};

// One GEMM launch of SPLIT, MERGED or DENSE.  Fitted to ~2500 stage tunings of the batch-1 layers
// (median relative error 5%, the picked tuning within 10% of the best one timed): a launch
// costs ~2.2 us however small plus 0.05 us per wavefront of its workgroups; a k-group ~0.065 us of issue per wavefront plus its MFMAs; the K x K
// stage pays for its gathered activation loads per pixel block; and the activation operand is
// re-read by every output-channel group, which is what makes taller register tiles (mb > 1) pay
// once there are many channel blocks -- charged as k-group loads per CU over the whole launch,
// more per load for a strided gather.
enum { G_LAUNCH, G_WAVE, G_KG, G_MFMA, G_CONV_B, G_REDUCE, G_ACT_1X1, G_ACT_CONV, G_TERMS };
const char *const kStageTermNames[G_TERMS] = {"launch", "wave", "kg", "mfma", "conv_b", "reduce", "act_1x1", "act_conv"};

const int kMb[3] = {1, 2, 4};

// Stage 1 of a one-launch kernel: rounds per wavefront, MFMA quads per k-group and unit, MB of x pulled
// per workgroup -- in the run-major form (`runs`) a unit is 16 runs of 4 pixels for mb1 channel blocks.
struct Stage1Work {
    int rounds, quads;
    double x_mb;
};
Stage1Work stage1_work(const TdcDims &d, const TdcFusedGeom &g, bool runs, int nw, int mb1, int pb)
{
    if (!runs) return {cdiv(cdiv(g.QB, pb) * (d.NB1 / mb1), nw), mb1 * pb, g.QB * 16.0 * d.C * 4e-6};
    const int rpr = tdc_runs_per_row(d.W, d.Wo, g.TW, d.K, d.stride, d.pad);
    return {cdiv(cdiv(g.QH * rpr, 16) * (d.NB1 / mb1), nw), 4 * mb1, g.QH * rpr * 16.0 * d.C * 1e-6};
}

inline double dot(const double *coef, const double *terms, int n)
{
    double t = 0.0;
    for (int i = 0; i < n; ++i) t += coef[i] * terms[i];
    return t;
}

// `by_registers`: residency from the register footprint of the unit (throughput fit) or from the wavefront slots
void fused_terms(double (&f)[F_TERMS], bool by_registers, const TdcDims &d, const TdcDeviceInfo &dev, const TdcFusedGeom &g,
                 bool runs, int nw, int mb1, int mb2, int mb3, int pb)
{
    const int KG2 = d.K * d.K * d.NB1, KG3 = d.NB2;
    const Stage1Work s1 = stage1_work(d, g, runs, nw, mb1, pb);
    const int r2 = cdiv(cdiv(g.PBk, pb) * (d.NB2 / mb2), nw);
    const int r3 = cdiv(cdiv(g.PBk, pb) * (d.NB3 / mb3), nw);
    const long wgs = (long)g.tiles_x * g.tiles_y * d.B;
    // register tiles of 1, 2, 4+ blocks leave room for 4, 3, 2 wavefronts per SIMD (kernel resource usage of the instances)
    const int unit = mb1 * pb, wps = !by_registers ? kWavesPerCu / 4 : unit == 1 ? 4 : unit == 2 ? 3 : 2;
    const int resident = resident_wgs(dev, g.lds_bytes, nw, wps);
    const int per_cu = (int)std::min<long>(resident, (wgs + dev.cus - 1) / dev.cus);
    const double rounds = std::ceil((double)wgs / ((double)dev.cus * resident));
    const double share = std::max(1.0, per_cu * nw / 4.0);
    const bool wl = g.weights_in_lds;
    const double w_kb = wl ? (double)(d.NB2 * KG2 + d.NB3 * KG3) : 0.0;
    for (double &v : f) v = 0.0;
    f[F_LAUNCH] = 1.0;
    f[runs ? F_S1R_UNIT : F_S1_UNIT] = rounds * s1.rounds;
    f[runs ? F_S1R_KG : F_S1_KG] = rounds * s1.rounds * d.KG1;
    f[runs ? F_S1R_MFMA : F_S1_MFMA] = rounds * s1.rounds * d.KG1 * s1.quads * share;
    f[wl ? F_S2_KG_LDS : F_S2_KG_GLB] = rounds * r2 * KG2;
    f[F_S2_MFMA] = rounds * r2 * KG2 * mb2 * pb * share;
    f[F_S3_UNIT] = rounds * r3;
    f[wl ? F_S3_KG_LDS : F_S3_KG_GLB] = rounds * r3 * KG3;
    f[F_S3_MFMA] = rounds * r3 * KG3 * mb3 * pb * share;
    f[F_W_KB] = rounds * w_kb * per_cu;
    f[d.nhwc ? F_X_MB_NHWC : runs ? F_X_MB_RUNS : F_X_MB_NCHW] = rounds * per_cu * s1.x_mb;
    f[d.nhwc ? F_Y_MB_NHWC : F_Y_MB_NCHW] = rounds * per_cu * g.PBk * 16.0 * d.N * 4e-6;
    if (!d.nhwc) {
        if (!runs) f[F_X_ROWS] = rounds * per_cu * g.QH * d.C * 1e-3;
        f[F_Y_ROWS] = rounds * per_cu * g.TH * d.N * 1e-3;
    }
}

double fused_us(bool throughput, const TdcDims &d, const TdcDeviceInfo &dev, const TdcFusedGeom &g, bool runs, int nw,
                int mb1, int mb2, int mb3, int pb)
{
    double f[F_TERMS];
    fused_terms(f, throughput, d, dev, g, runs, nw, mb1, mb2, mb3, pb);
    return dot(throughput ? kFusedThroughputCoef : kFusedLatencyCoef, f, F_TERMS);
}

struct FusedChoice {
    double us = 1e300;
    int th = 0, tw = 0, nw = 0, mb1 = 0, mb2 = 0, mb3 = 0, pb = 0;
};

FusedChoice best_fused(const TdcDims &d, const TdcDeviceInfo &dev, const tdc_tuning &forced)
{
    const bool throughput = (long)d.B * d.Ho * d.Wo >= 16L * dev.cus;
    const bool runs = tdc_runs_apply(d, dev.cus);
    FusedChoice best;
    const int th_lo = forced.tile_h ? forced.tile_h : 1, th_hi = forced.tile_h ? forced.tile_h : std::min(d.Ho, 16);
    const int tw_lo = forced.tile_w ? forced.tile_w : 1, tw_hi = forced.tile_w ? forced.tile_w : std::min(d.Wo, 32);
    for (int th = th_lo; th <= th_hi; ++th)
        for (int tw = tw_lo; tw <= tw_hi; ++tw) {
            if (th * tw > 512) continue;
            if (!forced.tile_w && tw < std::min(d.Wo, 4)) continue;   // keep rows long enough to coalesce
            const TdcFusedGeom g = tdc_fused_geometry(d, th, tw, dev.lds_per_wg);
            if ((long)g.lds_bytes > dev.lds_per_wg) continue;
            for (int nw : {8, 4, 2, 1}) {   // at equal estimate the first wins: more wavefronts hide more latency
                if (forced.waves[0] && nw != forced.waves[0]) continue;
                for (int pb : {1, 2})
                    for (int mb1 : kMb)
                        for (int mb2 : kMb)
                            for (int mb3 : kMb) {
                                if (forced.mb[0] && mb1 != forced.mb[0]) continue;
                                if (forced.mb[1] && mb2 != forced.mb[1]) continue;
                                if (forced.mb[2] && mb3 != forced.mb[2]) continue;
                                if (forced.pb[0] && pb != forced.pb[0]) continue;
                                if (d.NB1 % mb1 || d.NB2 % mb2 || d.NB3 % mb3) continue;   // whole register tiles only
                                if (!tdc_fused_unit_supported(mb1, mb2, mb3, pb)) continue;
                                const double us = fused_us(throughput, d, dev, g, runs, nw, mb1, mb2, mb3, pb);
                                if (us < best.us) {
                                    best.us = us;
                                    best.th = th; best.tw = tw; best.nw = nw;
                                    best.mb1 = mb1; best.mb2 = mb2; best.mb3 = mb3; best.pb = pb;
                                }
                            }
            }
        }
    return best;
}

// CHAIN: stage 1 as in FUSED; then every wavefront runs stages 2 and 3 for its own pixel-block
// groups: rounds23 * (KG2 * (kg + blk2 * NB2*PB*share) + NB3 * (nb + blk3 * NB2*PB*share)).  This
// variant serves the throughput regime, so the estimate also charges the bytes a CU pulls and
// pushes (input tile incl. halo, output tile) and the scalar-store path taken when tile or image
// width is not a multiple of 4, and, in NCHW, the number of row segments a CU reads and writes
// (tiles that span whole image rows move longer runs).  Fitted to ~12600 tunings of eight batch-8 to
// batch-64 layers, the NCHW ones timed with both forms of stage 1 (median relative error 9%).
enum {
    C_LAUNCH, C_S1_UNIT, C_S1_KG, C_S1_MFMA, C_S1R_UNIT, C_S1R_KG, C_S1R_MFMA,
    C_KG2_LDS, C_KG2_GLB, C_BLK2,                  // stage 2 per k-group (weights in LDS / streamed), per MFMA quad x pipe share
    C_NB3_LDS, C_BLK3,                             // stage 3 per output block with weights in LDS, per MFMA quad
    C_W_KB, C_X_MB_NCHW, C_X_MB_NHWC, C_X_MB_RUNS, C_Y_MB, C_X_ROWS, C_Y_ROWS,
    C_NOVEC,                                       // per output-channel block and pixel block stored with 4-byte stores
    C_TERMS
};
const char *const kChainTermNames[C_TERMS] = {"launch", "s1_unit", "s1_kg", "s1_mfma", "s1r_unit", "s1r_kg", "s1r_mfma",
                                              "kg2_lds", "kg2_glb", "blk2", "nb3_lds", "blk3", "w_kb", "x_mb_nchw", "x_mb_nhwc",
                                              "x_mb_runs", "y_mb", "x_rows", "y_rows", "novec"};

void chain_terms(double (&f)[C_TERMS], const TdcDims &d, const TdcDeviceInfo &dev, const TdcFusedGeom &g, bool runs, int nw,
                 int mb1, int pb, int *cu_waves)
{
    const int KG2 = d.K * d.K * d.NB1;
    const Stage1Work s1 = stage1_work(d, g, runs, nw, mb1, pb);
    const int r23 = cdiv(cdiv(g.PBk, pb), nw);
    const long wgs = (long)g.tiles_x * g.tiles_y * d.B;
    // Weights that fit in LDS are priced as staged there even where the kernel streams them instead (one group of
    // pixel blocks per wavefront): the coefficients were fitted on staged runs, and streaming is the cheaper of
    // the two in that case, so the ranking holds.
    const bool wl = g.weights_fit;
    const size_t w_bytes = (size_t)(d.NB2 * KG2 + d.NB3 * d.NB2) * 1024;
    const size_t lds_as_staged = g.lds_bytes + (g.weights_fit && !g.weights_in_lds ? w_bytes : 0);
    // two wavefronts per SIMD: what the instances needed when the table was fitted (they hold three or four since the
    // stage-1 width became a template parameter; the coefficients absorb the difference)
    const int resident = resident_wgs(dev, lds_as_staged, nw, 2);
    const int per_cu = (int)std::min<long>(resident, (wgs + dev.cus - 1) / dev.cus);
    *cu_waves = per_cu * nw;
    const double rounds = std::ceil((double)wgs / ((double)dev.cus * resident));
    const double share = std::max(1.0, per_cu * nw / 4.0);
    const double w_kb = wl ? (double)(d.NB2 * KG2 + d.NB3 * d.NB2) : 0.0;
    const bool vec = d.nhwc || (g.TW % 4 == 0 && d.Wo % 4 == 0);
    for (double &v : f) v = 0.0;
    f[C_LAUNCH] = 1.0;
    f[runs ? C_S1R_UNIT : C_S1_UNIT] = rounds * s1.rounds;
    f[runs ? C_S1R_KG : C_S1_KG] = rounds * s1.rounds * d.KG1;
    f[runs ? C_S1R_MFMA : C_S1_MFMA] = rounds * s1.rounds * d.KG1 * s1.quads * share;
    f[wl ? C_KG2_LDS : C_KG2_GLB] = rounds * r23 * KG2;
    f[C_BLK2] = rounds * r23 * KG2 * d.NB2 * pb * share;
    if (wl) f[C_NB3_LDS] = rounds * r23 * d.NB3;
    f[C_BLK3] = rounds * r23 * d.NB3 * d.NB2 * pb * share;
    if (!vec) f[C_NOVEC] = rounds * r23 * d.NB3 * pb;
    f[C_W_KB] = rounds * w_kb * per_cu;
    f[d.nhwc ? C_X_MB_NHWC : runs ? C_X_MB_RUNS : C_X_MB_NCHW] = rounds * per_cu * s1.x_mb;
    f[C_Y_MB] = rounds * per_cu * g.PBk * 16.0 * d.N * 4e-6;
    if (!d.nhwc) {
        if (!runs) f[C_X_ROWS] = rounds * per_cu * g.QH * d.C * 1e-3;
        f[C_Y_ROWS] = rounds * per_cu * g.TH * d.N * 1e-3;
    }
}

double chain_us(const TdcDims &d, const TdcDeviceInfo &dev, const TdcFusedGeom &g, bool runs, int nw, int mb1, int pb, int *cu_waves)
{
    double f[C_TERMS];
    chain_terms(f, d, dev, g, runs, nw, mb1, pb, cu_waves);
    return dot(kChainCoef, f, C_TERMS);
}

FusedChoice best_chain(const TdcDims &d, const TdcDeviceInfo &dev, const tdc_tuning &forced)
{
    const bool runs = tdc_runs_apply(d, dev.cus);
    FusedChoice best;
    int best_cu_waves = 0;
    long best_x_pixels = 0;
    const int th_lo = forced.tile_h ? forced.tile_h : 1, th_hi = forced.tile_h ? forced.tile_h : std::min(d.Ho, 16);
    const int tw_lo = forced.tile_w ? forced.tile_w : 1, tw_hi = forced.tile_w ? forced.tile_w : std::min(d.Wo, 32);
    for (int th = th_lo; th <= th_hi; ++th)
        for (int tw = tw_lo; tw <= tw_hi; ++tw) {
            if (th * tw > 512) continue;
            // NCHW: whole 16-byte quads where the image allows them (NHWC stores are 16 bytes whatever the tile)
            if (!forced.tile_w && !d.nhwc && d.Wo % 4 == 0 && tw % 4) continue;
            // The estimate is the same for one 8-wavefront workgroup per CU run twice and for two 4-wavefront ones run
            // together, and for 8 wavefronts with 16-pixel units against 4 with 32-pixel units.  Measured, more
            // wavefronts on the CU win, and at equal numbers the smaller workgroups (they fall out of step and
            // overlap their memory and arithmetic phases): ties go to more wavefronts, then to the tiling that reads the
            // fewest input pixels (the smallest halo overhead), then to workgroups of 4.
            for (int nw : {4, 8, 2, 1}) {
                if (forced.waves[0] && nw != forced.waves[0]) continue;
                for (int pb : {1, 2}) {
                    if (forced.pb[0] && pb != forced.pb[0]) continue;
                    const TdcFusedGeom g = tdc_chain_geometry(d, th, tw, nw, pb, dev.lds_per_wg);
                    if ((long)g.lds_bytes > dev.lds_per_wg) continue;
                    for (int mb1 : kMb) {
                        if (forced.mb[0] && mb1 != forced.mb[0]) continue;
                        if (d.NB1 % mb1 || !tdc_chain_supported(d.NB2, mb1, pb)) continue;
                        int cu_waves = 0;
                        const double us = chain_us(d, dev, g, runs, nw, mb1, pb, &cu_waves);
                        const bool tie = std::fabs(us - best.us) <= 1e-9 * us;
                        const long x_pixels = (long)g.tiles_x * g.tiles_y * g.Q;      // input pixels read per image, halos included
                        if ((!tie && us < best.us) || (tie && cu_waves > best_cu_waves) ||
                            (tie && cu_waves == best_cu_waves && x_pixels < best_x_pixels)) {
                            best_cu_waves = cu_waves;
                            best_x_pixels = x_pixels;
                            best.us = us;
                            best.th = th; best.tw = tw; best.nw = nw;
                            best.mb1 = mb1; best.mb2 = 1; best.mb3 = 1; best.pb = pb;
                        }
                    }
                }
            }
        }
    // One channel block per stage-1 unit issues the loads of the input tile once per block.  Two blocks per unit were
    // 2-17 % faster at the same tile in every NHWC sweep timed, and in the NCHW ones from 64 output pixels per compute
    // unit (below that, 12-16 % slower), which the fitted stage-1 terms do not reproduce: the choice of tile stands,
    // the unit is widened afterwards.
    const bool widen = d.nhwc || (long)d.B * d.Ho * d.Wo >= 64L * dev.cus;
    if (!forced.mb[0] && widen && best.mb1 == 1 && d.NB1 % 2 == 0 && tdc_chain_supported(d.NB2, 2, best.pb)) best.mb1 = 2;
    return best;
}

// FUSED_MERGED: stage 1 as in FUSED (dealt over nw wavefronts), then every wavefront runs its
// slice of the merged convolution out of registers and LDS.  Fitted to ~6600 tunings of 27 batch-1
// layer shapes in both activation layouts (median relative error 8%; the picked tuning on average
// 5% behind the best one timed): per stage-1 unit 0.22 us plus its k-groups and MFMAs, 0.08 us per
// weight fragment and pixel block of the tail, 0.45 us for a cross-slice sum, the bytes of x a CU
// pulls (input tile with halo, once per workgroup; dearer in NCHW, where they arrive as 4-byte
// loads), and a dispatch term per 256 workgroups -- the recomputation of stage 1 by every
// output-channel group shows up there and in the x bytes.
enum { M_LAUNCH, M_S1_UNIT, M_S1_KG, M_S1_MFMA, M_FRAG, M_REDUCE, M_X_MB_NCHW, M_X_MB_NHWC, M_WGS, M_TERMS };
const char *const kFmTermNames[M_TERMS] = {"launch", "s1_unit", "s1_kg", "s1_mfma", "frag", "reduce", "x_mb_nchw", "x_mb_nhwc", "wgs"};

struct FmChoice {
    double us = 1e300;
    bool calibrated = false;      // found inside the region the coefficients were fitted on
    int th = 0, tw = 0, nw = 0, mb1 = 0, nbg = 0;
};

void fm_terms(double (&f)[M_TERMS], const TdcDims &d, const TdcDeviceInfo &dev, const TdcFusedGeom &g, int nw, int mb1, int nbg)
{
    const int KG2 = d.K * d.K * d.NB1, ks = nw / nbg;
    const long wgs = (long)g.tiles_x * g.tiles_y * (d.NB3 / nbg) * d.B;
    const int resident = std::max(1, std::min({(int)(dev.lds_per_wg / std::max<size_t>(g.lds_bytes, 1)), kWavesPerCu / nw, 8}));
    const int per_cu = (int)std::min<long>(resident, (wgs + dev.cus - 1) / dev.cus);
    const double rounds = std::ceil((double)wgs / ((double)dev.cus * resident));
    const double share = std::max(1.0, per_cu * nw / 4.0);
    const int r1 = cdiv(g.QB * (d.NB1 / mb1), nw);
    const int frags = cdiv(KG2, ks);
    for (double &v : f) v = 0.0;
    f[M_LAUNCH] = 1.0;
    f[M_S1_UNIT] = rounds * r1;
    f[M_S1_KG] = rounds * r1 * d.KG1;
    f[M_S1_MFMA] = rounds * r1 * d.KG1 * mb1 * share;
    f[M_FRAG] = rounds * g.PBk * frags * share;
    if (ks > 1) f[M_REDUCE] = rounds * g.PBk;
    f[d.nhwc ? M_X_MB_NHWC : M_X_MB_NCHW] = rounds * per_cu * g.QB * 16.0 * d.C * 4e-6;
    f[M_WGS] = wgs / 256.0;
}

double fm_us(const TdcDims &d, const TdcDeviceInfo &dev, const TdcFusedGeom &g, int nw, int mb1, int nbg)
{
    double f[M_TERMS];
    fm_terms(f, d, dev, g, nw, mb1, nbg);
    return dot(kFmCoef, f, M_TERMS);
}

FmChoice best_fm(const TdcDims &d, const TdcDeviceInfo &dev, const tdc_tuning &forced)
{
    FmChoice best;
    const int ks_min = cdiv(d.K * d.K * d.NB1, 9);   // a wavefront holds nine weight fragments
    const int th_lo = forced.tile_h ? forced.tile_h : 1, th_hi = forced.tile_h ? forced.tile_h : std::min(d.Ho, 8);
    const int tw_lo = forced.tile_w ? forced.tile_w : 1, tw_hi = forced.tile_w ? forced.tile_w : std::min(d.Wo, 32);
    // pass 0: the calibrated region only; pass 1 (shapes that have no tuning there): anything launchable
    for (int pass = 0; pass < 2 && best.us >= 1e299; ++pass)
    for (int th = th_lo; th <= th_hi; ++th)
        for (int tw = tw_lo; tw <= tw_hi; ++tw) {
            if (th * tw > 64) continue;
            if (!forced.tile_w && tw < std::min(d.Wo, 4)) continue;
            for (int nbg = 1; nbg <= 8; ++nbg)
                for (int nw = nbg; nw <= 8; nw += nbg)
                    for (int mb1 : kMb) {
                        if (forced.waves[0] && nw != forced.waves[0]) continue;
                        if (forced.mb[0] && mb1 != forced.mb[0]) continue;
                        if (forced.mb[1] && nbg != forced.mb[1]) continue;
                        if (!tdc_fm_supported(d, th, tw, nw, mb1, nbg)) continue;
                        // the calibrated region: 2, 4 or 8 wavefronts, as few contraction slices as the
                        // register budget allows, or twice that
                        const int ks = nw / nbg;
                        if (pass == 0 && !forced.waves[0] && nw != 2 && nw != 4 && nw != 8) continue;
                        if (pass == 0 && !forced.waves[0] && !forced.mb[1] && ks != ks_min && ks != 2 * ks_min) continue;
                        const TdcFusedGeom g = tdc_fm_geometry(d, th, tw, nw, nbg);
                        if ((long)g.lds_bytes > dev.lds_per_wg) continue;
                        const double us = fm_us(d, dev, g, nw, mb1, nbg);
                        if (us < best.us) {
                            best.us = us;
                            best.th = th; best.tw = tw; best.nw = nw; best.mb1 = mb1; best.nbg = nbg;
                            best.calibrated = pass == 0;
                        }
                    }
        }
    return best;
}

struct StageChoice {
    double us = 1e300;
    int mb = 1, pb = 1, nw = 1;
};

// one GEMM launch: n_mblocks x n_pblocks output blocks per image, `kgroups` k-groups;
// conv_stride = 0 for a 1x1 stage, the stride for the K x K stage
void stage_terms(double (&f)[G_TERMS], const TdcDeviceInfo &dev, int batch, int n_mblocks, int n_pblocks, int kgroups, int mb, int pb,
                 int nw, int conv_stride)
{
    const long wgs = (long)(n_mblocks / mb) * cdiv(n_pblocks, pb) * batch;
    const int resident = std::max(1, std::min(kWavesPerCu / nw, 8));
    const int per_cu = (int)std::min<long>(resident, (wgs + dev.cus - 1) / dev.cus);
    const double rounds = std::ceil((double)wgs / ((double)dev.cus * resident));
    const double share = std::max(1.0, per_cu * nw / 4.0);
    const int kgw = cdiv(kgroups, nw);
    const double act_loads = (double)batch * (n_mblocks / mb) * n_pblocks * kgroups / dev.cus;
    for (double &v : f) v = 0.0;
    f[G_LAUNCH] = 1.0;
    f[G_WAVE] = rounds * nw;
    f[G_KG] = rounds * kgw;
    f[G_MFMA] = rounds * kgw * mb * pb * share;
    if (conv_stride) f[G_CONV_B] = rounds * kgw * pb;
    if (nw > 1) f[G_REDUCE] = rounds * mb * pb;
    f[conv_stride ? G_ACT_CONV : G_ACT_1X1] = act_loads * (conv_stride ? conv_stride : 1);
}

// The dense layer (tdc_conv_dense: one GEMM launch that writes the layer's y) has a table of its own: the terms of a GEMM
// stage, fitted to launches that carry an epilogue as the layers of the bottleneck networks do, and the outputs a thread
// owns -- 4 * mb * pb per lane when a wavefront works alone, 4 * mb * pb / nw when nw wavefronts sum through LDS and
// share the stores.  In NCHW every one of them is a 4-byte store (and with a residual a 4-byte load before it), which
// the stage table, calibrated on launches without an epilogue, had no term for: it took 1-wavefront units of four
// channel blocks for the 64 -> 256 expansion at 56x56 (8.0 us, where two wavefronts on one block run in 5.8 us).
enum { D_Y_NCHW = G_TERMS, D_Y_NHWC, D_TERMS };
const char *const kDenseTermNames[D_TERMS] = {"launch", "wave", "kg", "mfma", "conv_b", "reduce", "act_1x1", "act_conv", "y_nchw", "y_nhwc"};

void dense_terms(double (&f)[D_TERMS], const TdcDeviceInfo &dev, int batch, int n_mblocks, int n_pblocks, int kgroups, int mb, int pb,
                 int nw, int conv_stride, bool nhwc)
{
    double g[G_TERMS];
    stage_terms(g, dev, batch, n_mblocks, n_pblocks, kgroups, mb, pb, nw, conv_stride);
    for (int i = 0; i < G_TERMS; ++i) f[i] = g[i];
    const double per_thread = 4.0 * mb * pb / nw;
    f[D_Y_NCHW] = nhwc ? 0.0 : per_thread;
    f[D_Y_NHWC] = nhwc ? per_thread : 0.0;
}

// one GEMM launch: n_mblocks x n_pblocks output blocks per image, `kgroups` k-groups;
// conv_stride = 0 for a 1x1 stage, the stride for the K x K stage; `dense`: priced by the dense layer's table
StageChoice best_stage(const TdcDeviceInfo &dev, int batch, int n_mblocks, int n_pblocks, int kgroups, int fmb,
                       int fpb, int fnw, int conv_stride, bool dense = false, bool nhwc = false)
{
    StageChoice best;
    for (int mb : kMb)
        for (int pb : kMb)
            for (int nw : {1, 2, 3, 4, 6, 8}) {
                if (fmb && mb != fmb) continue;
                if (fpb && pb != fpb) continue;
                if (fnw && nw != fnw) continue;
                // 3 and 6 wavefronts are launchable and never chosen: they leave the four SIMDs of a compute unit with
                // unequal shares (2, 2, 1, 1), and in every sweep the next power of two was as fast or faster (6 against
                // 8 wavefronts: +0.5 to +1.0 us on the rank-40 and rank-80 layers) while the fitted terms, smooth in
                // the wavefront count, put them in between
                if (!fnw && (nw == 3 || nw == 6)) continue;
                if (n_mblocks % mb) continue;         // whole register tiles only
                if (!fnw && nw > kgroups) continue;   // idle wavefronts are legal, just never chosen
                if ((size_t)nw * mb * pb * 1024 > 64 * 1024 && nw > 1) continue;
                double us;
                if (dense) {
                    double f[D_TERMS];
                    dense_terms(f, dev, batch, n_mblocks, n_pblocks, kgroups, mb, pb, nw, conv_stride, nhwc);
                    us = dot(kDenseCoef, f, D_TERMS);
                } else {
                    double f[G_TERMS];
                    stage_terms(f, dev, batch, n_mblocks, n_pblocks, kgroups, mb, pb, nw, conv_stride);
                    us = dot(kStageCoef, f, G_TERMS);
                }
                if (us < best.us) {
                    best.us = us;
                    best.mb = mb; best.pb = pb; best.nw = nw;
                }
            }
    return best;
}

}  // namespace

// The terms of the estimate for a fully specified tuning (see tdc_model_terms in tdc.h).
int tdc_select_terms(const TdcDims &d, const TdcDeviceInfo &dev, const tdc_tuning &t, double *terms, const char **names,
                     int max_terms, int *n_terms, const char **model)
{
    const bool runs = tdc_runs_apply(d, dev.cus);
    const auto emit = [&](const double *f, const char *const *nm, int n, const char *which) {
        if (n > max_terms) return (int)TDC_ERR_BAD_SHAPE;
        for (int i = 0; i < n; ++i) {
            terms[i] = f[i];
            if (names) names[i] = nm[i];
        }
        *n_terms = n;
        if (model) *model = which;
        return (int)TDC_OK;
    };
    if (t.variant == TDC_VARIANT_FUSED) {
        const bool throughput = (long)d.B * d.Ho * d.Wo >= 16L * dev.cus;
        const TdcFusedGeom g = tdc_fused_geometry(d, t.tile_h, t.tile_w, dev.lds_per_wg);
        double f[F_TERMS];
        fused_terms(f, throughput, d, dev, g, runs, t.waves[0], t.mb[0], t.mb[1], t.mb[2], t.pb[0]);
        return emit(f, kFusedTermNames, F_TERMS, throughput ? "fused_throughput" : "fused_latency");
    }
    if (t.variant == TDC_VARIANT_CHAIN) {
        const TdcFusedGeom g = tdc_chain_geometry(d, t.tile_h, t.tile_w, t.waves[0], t.pb[0], dev.lds_per_wg);
        double f[C_TERMS];
        int cu_waves = 0;
        chain_terms(f, d, dev, g, runs, t.waves[0], t.mb[0], t.pb[0], &cu_waves);
        return emit(f, kChainTermNames, C_TERMS, "chain");
    }
    if (t.variant == TDC_VARIANT_FUSED_MERGED) {
        const TdcFusedGeom g = tdc_fm_geometry(d, t.tile_h, t.tile_w, t.waves[0], t.mb[1]);
        double f[M_TERMS];
        fm_terms(f, d, dev, g, t.waves[0], t.mb[0], t.mb[1]);
        return emit(f, kFmTermNames, M_TERMS, "fused_merged");
    }
    if (t.variant == TDC_VARIANT_SPLIT || t.variant == TDC_VARIANT_MERGED || t.variant == TDC_VARIANT_MERGED_XCD ||
        t.variant == TDC_VARIANT_DENSE) {
        // the launches of a call share one set of coefficients, so their terms add up
        const int pb_in = cdiv(d.H * d.W, 16), pb_out = cdiv(d.Ho * d.Wo, 16), KG2 = d.K * d.K * d.NB1;
        double f[G_TERMS], sum[G_TERMS] = {0};
        const auto add = [&](int n_mblocks, int n_pblocks, int kgroups, int st, int conv_stride) {
            stage_terms(f, dev, d.B, n_mblocks, n_pblocks, kgroups, t.mb[st], t.pb[st], t.waves[st], conv_stride);
            for (int i = 0; i < G_TERMS; ++i) sum[i] += f[i];
        };
        if (t.variant == TDC_VARIANT_DENSE) {
            double fd[D_TERMS];
            dense_terms(fd, dev, d.B, d.NB2, pb_out, KG2, t.mb[1], t.pb[1], t.waves[1], d.stride, d.nhwc != 0);
            return emit(fd, kDenseTermNames, D_TERMS, "dense");
        } else {
            add(d.NB1, pb_in, d.KG1, 0, 0);
            if (t.variant == TDC_VARIANT_MERGED || t.variant == TDC_VARIANT_MERGED_XCD) {
                add(d.NB3, pb_out, KG2, 1, d.stride);
            } else {
                add(d.NB2, pb_out, KG2, 1, d.stride);
                add(d.NB3, pb_out, d.NB2, 2, 0);
            }
        }
        return emit(sum, kStageTermNames, G_TERMS, "stage");
    }
    return TDC_ERR_BAD_TUNING;
}

// MERGED_XCD: as many wavefronts per 16x16 unit as still give every unit a team in one pass -- stage 1 over the 32
// workgroups an XCD can have, the merged GEMM over all 256 -- and never more than the unit has k-groups.
struct XcdChoice {
    int tw1, tw2;
    bool one_pass;
};
static XcdChoice best_xcd(const TdcDims &d, const tdc_tuning &forced)
{
    const long n1 = (long)d.B * d.NB1 * cdiv(d.H * d.W, 16), n2 = (long)d.B * d.NB3 * cdiv(d.Ho * d.Wo, 16);
    const int kg1 = d.KG1, kg2 = d.K * d.K * d.NB1;
    XcdChoice c{1, 1, false};
    for (int tw = 8; tw >= 1; tw /= 2)
        if (tw <= kg1 && n1 <= 32L * (8 / tw)) { c.tw1 = tw; break; }
    for (int tw = 8; tw >= 1; tw /= 2)
        if (tw <= kg2 && n2 <= 256L * (8 / tw)) { c.tw2 = tw; break; }
    c.one_pass = n1 <= 32L * (8 / c.tw1) && n2 <= 256L * (8 / c.tw2);
    if (forced.waves[0]) c.tw1 = forced.waves[0];
    if (forced.waves[1]) c.tw2 = forced.waves[1];
    return c;
}
int tdc_select(const TdcDims &d, const TdcDeviceInfo &dev, tdc_tuning *t, double *model_us)
{
    if (model_us) *model_us = 0.0;
    const tdc_tuning forced = *t;
    if (forced.variant == TDC_VARIANT_NAIVE) return TDC_OK;
    if (forced.variant == TDC_VARIANT_DENSE) {
        // the stage-2 kernel on the layer's own channels: `d` has R1 = C and R2 = N
        const StageChoice c = best_stage(dev, d.B, d.NB2, cdiv(d.Ho * d.Wo, 16), d.K * d.K * d.NB1, forced.mb[1],
                                         forced.pb[1], forced.waves[1], d.stride, true, d.nhwc != 0);
        if (c.us >= 1e299) return TDC_ERR_BAD_TUNING;
        t->tile_h = t->tile_w = 0;
        for (int i = 0; i < 3; ++i) {
            t->mb[i] = c.mb; t->pb[i] = c.pb; t->waves[i] = c.nw;
        }
        if (model_us) *model_us = c.us;
        return TDC_OK;
    }
    if (forced.variant == TDC_VARIANT_FUSED_MERGED) {
        const FmChoice c = best_fm(d, dev, forced);
        if (c.us >= 1e299) return TDC_ERR_BAD_TUNING;
        t->tile_h = c.th; t->tile_w = c.tw;
        t->waves[0] = t->waves[1] = t->waves[2] = c.nw;
        t->mb[0] = c.mb1; t->mb[1] = c.nbg; t->mb[2] = 1;
        t->pb[0] = t->pb[1] = t->pb[2] = 1;
        if (model_us) *model_us = c.us;
        return TDC_OK;
    }
    if (forced.variant == TDC_VARIANT_MERGED) {
        const StageChoice a = best_stage(dev, d.B, d.NB1, cdiv(d.H * d.W, 16), d.KG1, forced.mb[0], forced.pb[0], forced.waves[0], 0);
        const StageChoice b = best_stage(dev, d.B, d.NB3, cdiv(d.Ho * d.Wo, 16), d.K * d.K * d.NB1, forced.mb[1], forced.pb[1],
                                         forced.waves[1], d.stride);
        if (a.us >= 1e299 || b.us >= 1e299) return TDC_ERR_BAD_TUNING;
        t->tile_h = t->tile_w = 0;
        t->mb[0] = a.mb; t->pb[0] = a.pb; t->waves[0] = a.nw;
        t->mb[1] = t->mb[2] = b.mb; t->pb[1] = t->pb[2] = b.pb; t->waves[1] = t->waves[2] = b.nw;
        if (model_us) *model_us = a.us + b.us;
        return TDC_OK;
    }
    if (forced.variant == TDC_VARIANT_MERGED_XCD) {
        for (int i = 0; i < 2; ++i)
            if (forced.mb[i] > 1 || forced.pb[i] > 1) return TDC_ERR_BAD_TUNING;   // units are single 16x16 blocks
        XcdChoice c = best_xcd(d, forced);
        t->tile_h = t->tile_w = 0;
        for (int i = 0; i < 3; ++i) t->mb[i] = t->pb[i] = 1;
        t->waves[0] = c.tw1; t->waves[1] = t->waves[2] = c.tw2;
        if (model_us) {
            const StageChoice a = best_stage(dev, d.B, d.NB1, cdiv(d.H * d.W, 16), d.KG1, 1, 1, c.tw1, 0);
            const StageChoice b = best_stage(dev, d.B, d.NB3, cdiv(d.Ho * d.Wo, 16), d.K * d.K * d.NB1, 1, 1, c.tw2, d.stride);
            *model_us = a.us < 1e299 && b.us < 1e299 ? a.us + b.us : 0.0;   // measured within 3 % of MERGED's two launches
        }
        return TDC_OK;
    }
    if (forced.variant == TDC_VARIANT_CHAIN) {
        const FusedChoice c = best_chain(d, dev, forced);
        if (c.us >= 1e299) return TDC_ERR_BAD_TUNING;
        t->tile_h = c.th; t->tile_w = c.tw;
        t->waves[0] = t->waves[1] = t->waves[2] = c.nw;
        t->mb[0] = c.mb1; t->mb[1] = 1; t->mb[2] = 1;
        t->pb[0] = t->pb[1] = t->pb[2] = c.pb;
        if (model_us) *model_us = c.us;
        return TDC_OK;
    }

    FusedChoice f;
    if (forced.variant == TDC_VARIANT_AUTO || forced.variant == TDC_VARIANT_FUSED) f = best_fused(d, dev, forced);
    // output pixels alone give every CU a 16-pixel block: the throughput regime
    const bool pixels_fill_chip = (long)d.B * d.Ho * d.Wo >= 16L * dev.cus;
    // CHAIN keeps whole pixel blocks per wavefront and needs two 16-pixel blocks per CU to pay: below that FUSED,
    // which cuts the same tile along channels as well, won every sweep (batch 8 at 28x28, batch 32 at 14x14),
    // by 5-80%, while the two estimates are too close there to tell.
    const bool chain_pays = (long)d.B * d.Ho * d.Wo >= 32L * dev.cus;
    if (forced.variant == TDC_VARIANT_AUTO && chain_pays) {
        tdc_tuning free_choice = forced;
        const FusedChoice c = best_chain(d, dev, free_choice);
        // The two tables are fitted separately, and where the estimates are close FUSED's is the optimistic one (its
        // measured best lies 8-15 % further behind CHAIN's than estimated on the NCHW layers of the sweeps): FUSED has to
        // win by 7 %.
        if (0.93 * c.us < f.us) {
            t->variant = TDC_VARIANT_CHAIN;
            t->tile_h = c.th; t->tile_w = c.tw;
            t->waves[0] = t->waves[1] = t->waves[2] = c.nw;
            t->mb[0] = c.mb1; t->mb[1] = 1; t->mb[2] = 1;
            t->pb[0] = t->pb[1] = t->pb[2] = c.pb;
            if (model_us) *model_us = c.us;
            return TDC_OK;
        }
    }

    StageChoice s[3];
    double split_us = 1e300;
    if (forced.variant == TDC_VARIANT_AUTO || forced.variant == TDC_VARIANT_SPLIT) {
        const int pb_in = cdiv(d.H * d.W, 16), pb_out = cdiv(d.Ho * d.Wo, 16);
        s[0] = best_stage(dev, d.B, d.NB1, pb_in, d.KG1, forced.mb[0], forced.pb[0], forced.waves[0], 0);
        s[1] = best_stage(dev, d.B, d.NB2, pb_out, d.K * d.K * d.NB1, forced.mb[1], forced.pb[1], forced.waves[1], d.stride);
        s[2] = best_stage(dev, d.B, d.NB3, pb_out, d.NB2, forced.mb[2], forced.pb[2], forced.waves[2], 0);
        split_us = s[0].us + s[1].us + s[2].us;
    }

    // The merged forms (stage 3 folded into the core) against the others: only below the throughput
    // regime, where their extra MACs cost nothing and the saved launches count.  The one-launch
    // form's estimate is optimistic once the contraction is cut into three or more slices, so it
    // has to win by a margin, and only tunings inside its calibrated region are considered.
    if (forced.variant == TDC_VARIANT_AUTO && !pixels_fill_chip) {
        const StageChoice m2 = best_stage(dev, d.B, d.NB3, cdiv(d.Ho * d.Wo, 16), d.K * d.K * d.NB1, forced.mb[1], forced.pb[1],
                                          forced.waves[1], d.stride);
        tdc_tuning free_choice = forced;
        free_choice.mb[0] = free_choice.mb[1] = free_choice.mb[2] = 0;
        free_choice.waves[0] = 0;
        const FmChoice fm = best_fm(d, dev, free_choice);
        const int ks_min = cdiv(d.K * d.K * d.NB1, 9);   // slices the contraction needs at least
        const double fm_us = fm.calibrated ? fm.us * (ks_min >= 3 ? 1.20 : 1.05) : 1e300;
        if (fm_us < f.us && fm_us < split_us && fm_us < s[0].us + m2.us) {
            t->variant = TDC_VARIANT_FUSED_MERGED;
            t->tile_h = fm.th; t->tile_w = fm.tw;
            t->waves[0] = t->waves[1] = t->waves[2] = fm.nw;
            t->mb[0] = fm.mb1; t->mb[1] = fm.nbg; t->mb[2] = 1;
            t->pb[0] = t->pb[1] = t->pb[2] = 1;
            if (model_us) *model_us = fm.us;
            return TDC_OK;
        }
    }
    if (forced.variant == TDC_VARIANT_AUTO && !pixels_fill_chip) {
        const StageChoice m = best_stage(dev, d.B, d.NB3, cdiv(d.Ho * d.Wo, 16), d.K * d.K * d.NB1, forced.mb[1], forced.pb[1],
                                         forced.waves[1], d.stride);
        const double merged_us = s[0].us + m.us;
        if (merged_us < f.us && merged_us < split_us) {
            t->variant = TDC_VARIANT_MERGED;
            t->tile_h = t->tile_w = 0;
            t->mb[0] = s[0].mb; t->pb[0] = s[0].pb; t->waves[0] = s[0].nw;
            t->mb[1] = t->mb[2] = m.mb; t->pb[1] = t->pb[2] = m.pb; t->waves[1] = t->waves[2] = m.nw;
            if (model_us) *model_us = merged_us;
            return TDC_OK;
        }
    }

    int variant = forced.variant;
    if (variant == TDC_VARIANT_AUTO) {
        // The split estimate is calibrated on latency-bound launches (few workgroup rounds).  In the
        // throughput regime three launches that round-trip z1 and z2 through memory never beat the
        // fused kernels in the sweep, so the comparison is not trusted there.  Below it FUSED has to win by 8 %: where the
        // two estimates are that close the layer is a heavy one (many channels on few pixels), the fused latency table
        // ranks its own tunings badly there and the fused kernel measured 3-30 % behind SPLIT (512 channels on 7x7 at
        // batch 64: 50.2 against 38.3 us; 256 channels on 56x56: 17.9 against 17.4 us), 2 % ahead at best.
        variant = (f.us <= 0.92 * split_us || (pixels_fill_chip && f.us < 1e299)) ? TDC_VARIANT_FUSED : TDC_VARIANT_SPLIT;
    }
    if (variant == TDC_VARIANT_FUSED) {
        if (f.us >= 1e299) return TDC_ERR_BAD_TUNING;
        t->variant = TDC_VARIANT_FUSED;
        t->tile_h = f.th; t->tile_w = f.tw;
        t->waves[0] = t->waves[1] = t->waves[2] = f.nw;
        t->mb[0] = f.mb1; t->mb[1] = f.mb2; t->mb[2] = f.mb3;
        t->pb[0] = t->pb[1] = t->pb[2] = f.pb;
        if (model_us) *model_us = f.us;
        return TDC_OK;
    }
    if (split_us >= 1e299) return TDC_ERR_BAD_TUNING;
    t->variant = TDC_VARIANT_SPLIT;
    t->tile_h = t->tile_w = 0;
    for (int i = 0; i < 3; ++i) {
        t->mb[i] = s[i].mb; t->pb[i] = s[i].pb; t->waves[i] = s[i].nw;
    }
    if (model_us) *model_us = split_us;
    return TDC_OK;
}
