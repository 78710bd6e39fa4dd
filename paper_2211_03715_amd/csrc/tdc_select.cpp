// Tile / launch-parameter selector (host only).
//
// The paper picks its (TH, TW, TC) tile with an analytical model (section 5.3-5.5): a
// compute-latency term from the number of thread-block waves, then the smallest memory
// volume among the best few percent.  That model is built around one-thread-per-output-
// channel blocks on an NVIDIA SM; this one keeps the idea -- enumerate every tiling, score
// it with a closed-form latency estimate, no search on the device -- with terms that
// describe this library's kernels on CDNA4: MFMA issue cycles per SIMD, bytes pulled
// through a CU's L2 port, a fixed latency per dependent phase, and rounds of workgroups
// over the compute units.  All times are in shader clocks.
#include <algorithm>
#include <climits>
#include <cmath>

#include "tdc_internal.h"

namespace {

struct Machine {
    double mfma_clk = 32.0;       // issue cycles of one v_mfma_f32_16x16x4_f32 on its SIMD
    double l2_bytes_clk = 64.0;   // bytes per clock one CU pulls from L2
    double phase_lat = 900.0;     // exposed load latency at the start of a dependent phase
    double kgroup_ovh = 24.0;     // address / wait overhead per 16-wide k-group per unit
    double launch = 4500.0;       // one dependent kernel launch on a stream (about 1.9 us at 2.4 GHz)
    double wg_start = 1500.0;     // workgroup dispatch + first instruction fetch
};

inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// time of one GEMM-like phase executed by `nw` wavefronts of one workgroup
double phase_cycles(const Machine &m, int n_mblocks, int n_pblocks, int kgroups, int mb, int pb, int nw,
                    int ksplit)
{
    const int units = cdiv(n_mblocks, mb) * cdiv(n_pblocks, pb);
    const int waves_per_unit = ksplit;                        // wavefronts sharing one unit's contraction
    const int unit_slots = std::max(1, nw / waves_per_unit);
    const int rounds = cdiv(units, unit_slots);
    const double kg_per_wave = std::ceil((double)kgroups / ksplit);
    const double simd_share = std::max(1.0, nw / 4.0);        // wavefronts per SIMD issue in turn
    const double per_unit = kg_per_wave * (4.0 * mb * pb * m.mfma_clk * simd_share + m.kgroup_ovh);
    return m.phase_lat + rounds * per_unit;
}

struct FusedChoice {
    double cycles = 1e300;
    int th = 0, tw = 0, nw = 0, mb1 = 0, mb2 = 0, mb3 = 0, pb = 0;
};

const int kFusedMenu[][4] = {{1, 1, 1, 1}, {1, 1, 2, 1}, {2, 2, 2, 1}, {2, 2, 4, 1}, {4, 4, 4, 1},
                             {1, 1, 2, 2}, {2, 2, 2, 2}, {2, 2, 4, 2}, {4, 4, 4, 2}, {1, 1, 1, 2}};

double fused_cycles(const Machine &m, const TdcDims &d, const TdcDeviceInfo &dev, int th, int tw, int nw,
                    const int *menu, size_t *lds_out)
{
    TdcFusedGeom g = tdc_fused_geometry(d, th, tw, dev.lds_per_wg);
    *lds_out = g.lds_bytes;
    if ((long)g.lds_bytes > dev.lds_per_wg) return 1e300;
    const int KG2 = d.K * d.K * d.NB1;
    double t = m.wg_start;
    t += phase_cycles(m, d.NB1, g.QB, d.KG1, menu[0], menu[3], nw, 1);
    t += phase_cycles(m, d.NB2, g.PBk, KG2, menu[1], menu[3], nw, 1);
    t += phase_cycles(m, d.NB3, g.PBk, d.NB2, menu[2], menu[3], nw, 1);
    // bytes through the CU's L2 port: x tile once per stage-1 m-group, weights once per unit column
    const double wbytes = 1024.0 * ((double)d.NB1 * d.KG1 * cdiv(g.QB, menu[3]) +
                                    (double)d.NB2 * KG2 * cdiv(g.PBk, menu[3]) +
                                    (double)d.NB3 * d.NB2 * cdiv(g.PBk, menu[3]));
    const double xbytes = 4.0 * g.Q * d.C * cdiv(d.NB1, menu[0]);
    t = std::max(t, m.wg_start + (wbytes + xbytes) / m.l2_bytes_clk);
    const long wgs = (long)g.tiles_x * g.tiles_y * d.B;
    const int per_cu = std::max(1, std::min((int)(dev.lds_per_wg / std::max<size_t>(g.lds_bytes, 1)), 8 / std::max(1, nw / 4)));
    const double rounds = std::ceil((double)wgs / ((double)dev.cus * per_cu));
    // co-resident workgroups share the CU's SIMDs: charge the MFMA part once per resident group
    const double resident = std::min<double>(per_cu, std::ceil((double)wgs / dev.cus));
    return m.launch + rounds * t * std::max(1.0, resident * nw / 4.0) / std::max(1.0, nw / 4.0);
}

FusedChoice best_fused(const Machine &m, const TdcDims &d, const TdcDeviceInfo &dev, const tdc_tuning &forced)
{
    FusedChoice best;
    const int th_lo = forced.tile_h ? forced.tile_h : 1, th_hi = forced.tile_h ? forced.tile_h : std::min(d.Ho, 16);
    const int tw_lo = forced.tile_w ? forced.tile_w : 1, tw_hi = forced.tile_w ? forced.tile_w : std::min(d.Wo, 32);
    for (int th = th_lo; th <= th_hi; ++th)
        for (int tw = tw_lo; tw <= tw_hi; ++tw) {
            if (th * tw > 512) continue;
            if (!forced.tile_w && tw < std::min(d.Wo, 7)) continue;   // keep rows long enough to coalesce
            for (int nw : {1, 2, 4, 8}) {
                if (forced.waves[0] && nw != forced.waves[0]) continue;
                for (const auto &menu : kFusedMenu) {
                    if (forced.mb[0] && menu[0] != forced.mb[0]) continue;
                    if (forced.mb[1] && menu[1] != forced.mb[1]) continue;
                    if (forced.mb[2] && menu[2] != forced.mb[2]) continue;
                    if (forced.pb[0] && menu[3] != forced.pb[0]) continue;
                    if (d.NB1 % menu[0] || d.NB2 % menu[1] || d.NB3 % menu[2]) continue;   // whole register tiles only
                    size_t lds;
                    double c = fused_cycles(m, d, dev, th, tw, nw, menu, &lds);
                    if (c < best.cycles) {
                        best.cycles = c;
                        best.th = th; best.tw = tw; best.nw = nw;
                        best.mb1 = menu[0]; best.mb2 = menu[1]; best.mb3 = menu[2]; best.pb = menu[3];
                    }
                }
            }
        }
    return best;
}

struct StageChoice {
    double cycles = 1e300;
    int mb = 1, pb = 1, nw = 1;
};

// one SPLIT stage: n_mblocks x n_pblocks output blocks per image, `kgroups` k-groups
StageChoice best_stage(const Machine &m, const TdcDeviceInfo &dev, int batch, int n_mblocks, int n_pblocks,
                       int kgroups, int fmb, int fpb, int fnw)
{
    StageChoice best;
    for (int mb : {1, 2, 4})
        for (int pb : {1, 2, 4})
            for (int nw : {1, 2, 3, 4, 6, 8}) {
                if (fmb && mb != fmb) continue;
                if (fpb && pb != fpb) continue;
                if (fnw && nw != fnw) continue;
                if (n_mblocks % mb) continue;         // whole register tiles only
                if (!fnw && nw > kgroups) continue;   // idle wavefronts are legal, just never chosen
                if ((size_t)nw * mb * pb * 1024 > 64 * 1024 && nw > 1) continue;
                const long wgs = (long)cdiv(n_mblocks, mb) * cdiv(n_pblocks, pb) * batch;
                double t = m.wg_start + phase_cycles(m, mb, pb, kgroups, mb, pb, nw, nw);
                if (nw > 1) t += 200.0 + 8.0 * mb * pb;                       // LDS reduction
                const double bytes = 1024.0 * mb * kgroups + 1024.0 * pb * kgroups;   // operands of one unit
                t = std::max(t, m.wg_start + bytes / m.l2_bytes_clk);
                const int per_cu = std::max(1, 32 / nw);
                const double resident = std::min<double>(per_cu, std::ceil((double)wgs / dev.cus));
                const double rounds = std::ceil((double)wgs / ((double)dev.cus * per_cu));
                const double c = rounds * t * std::max(1.0, resident * nw / 4.0) / std::max(1.0, nw / 4.0);
                if (c < best.cycles) {
                    best.cycles = c;
                    best.mb = mb; best.pb = pb; best.nw = nw;
                }
            }
    return best;
}

}  // namespace

int tdc_select(const TdcDims &d, const TdcDeviceInfo &dev, tdc_tuning *t)
{
    Machine m;
    const tdc_tuning forced = *t;
    if (forced.variant == TDC_VARIANT_NAIVE) return TDC_OK;

    FusedChoice f;
    if (forced.variant == TDC_VARIANT_AUTO || forced.variant == TDC_VARIANT_FUSED) f = best_fused(m, d, dev, forced);

    StageChoice s[3];
    double split_cycles = 1e300;
    if (forced.variant == TDC_VARIANT_AUTO || forced.variant == TDC_VARIANT_SPLIT) {
        const int pb_in = cdiv(d.H * d.W, 16), pb_out = cdiv(d.Ho * d.Wo, 16);
        s[0] = best_stage(m, dev, d.B, d.NB1, pb_in, d.KG1, forced.mb[0], forced.pb[0], forced.waves[0]);
        s[1] = best_stage(m, dev, d.B, d.NB2, pb_out, d.K * d.K * d.NB1, forced.mb[1], forced.pb[1], forced.waves[1]);
        s[2] = best_stage(m, dev, d.B, d.NB3, pb_out, d.NB2, forced.mb[2], forced.pb[2], forced.waves[2]);
        split_cycles = 3 * m.launch + s[0].cycles + s[1].cycles + s[2].cycles;
    }

    int variant = forced.variant;
    if (variant == TDC_VARIANT_AUTO) variant = (f.cycles <= split_cycles) ? TDC_VARIANT_FUSED : TDC_VARIANT_SPLIT;
    if (variant == TDC_VARIANT_FUSED) {
        if (f.cycles >= 1e299) return TDC_ERR_BAD_TUNING;
        t->variant = TDC_VARIANT_FUSED;
        t->tile_h = f.th; t->tile_w = f.tw;
        t->waves[0] = t->waves[1] = t->waves[2] = f.nw;
        t->mb[0] = f.mb1; t->mb[1] = f.mb2; t->mb[2] = f.mb3;
        t->pb[0] = t->pb[1] = t->pb[2] = f.pb;
        return TDC_OK;
    }
    if (split_cycles >= 1e299) return TDC_ERR_BAD_TUNING;
    t->variant = TDC_VARIANT_SPLIT;
    t->tile_h = t->tile_w = 0;
    for (int i = 0; i < 3; ++i) {
        t->mb[i] = s[i].mb; t->pb[i] = s[i].pb; t->waves[i] = s[i].nw;
    }
    return TDC_OK;
}
