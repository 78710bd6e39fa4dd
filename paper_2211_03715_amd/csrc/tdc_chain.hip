// CHAIN variant, host side: which shapes it covers, its tile geometry, and the launch.  The kernel is in
// tdc_chain_kernel.h; its instances are compiled in tdc_chain_mb1.hip, tdc_chain_mb2.hip and tdc_chain_mb4.hip.
#include "tdc_chain_kernel.h"

hipError_t tdc_launch_chain_mb1(const TdcChainArgs &, int, int, bool, int, dim3, dim3, size_t, hipStream_t, bool);
hipError_t tdc_launch_chain_mb2(const TdcChainArgs &, int, int, bool, int, dim3, dim3, size_t, hipStream_t, bool);
hipError_t tdc_launch_chain_mb4(const TdcChainArgs &, int, int, bool, int, dim3, dim3, size_t, hipStream_t, bool);

bool tdc_chain_supported(int nb2, int mb1, int pb)
{
    if (!(mb1 == 1 || mb1 == 2 || mb1 == 4) || !(pb == 1 || pb == 2)) return false;
#define TDC_X(N_) if (nb2 == N_) return true;
    TDC_CHAIN_NB2(TDC_X)
#undef TDC_X
    return false;
}

TdcFusedGeom tdc_chain_geometry(const TdcDims &d, int tile_h, int tile_w, int nw, int pb, int lds_limit)
{
    TdcFusedGeom g;
    g.TH = tile_h;
    g.TW = tile_w;
    g.QH = (tile_h - 1) * d.stride + d.K;
    g.QW = (tile_w - 1) * d.stride + d.K;
    g.Q = g.QH * g.QW;
    g.QB = (g.Q + 15) / 16;
    g.PBk = (tile_h * tile_w + 15) / 16;
    g.tiles_x = (d.Wo + tile_w - 1) / tile_w;
    g.tiles_y = (d.Ho + tile_h - 1) / tile_h;
    g.pitch1 = 16 * g.QB + 4;
    g.pitch2 = 0;
    const size_t tiles = (size_t)16 * d.NB1 * g.pitch1 * sizeof(float);
    const size_t weights = (tdc_packed_floats_core(d) + tdc_packed_floats_uout(d)) * sizeof(float);
    // The packed core and U_out go into LDS when they fit and a wavefront has more than one group of pixel
    // blocks to run them over.  With a single group every fragment is used once per wavefront: staging it
    // through LDS only adds the copy and the wait for it (measured 5-10% slower on batch-8 to batch-32 layers
    // of rank 24 and 32 than streaming the fragments from L2 two k-groups ahead).
    const int groups_per_wave = ((g.PBk + pb - 1) / pb + nw - 1) / nw;
    g.weights_fit = tiles + weights <= (size_t)lds_limit;
    g.weights_in_lds = g.weights_fit && groups_per_wave > 1;
    g.lds_bytes = tiles + (g.weights_in_lds ? weights : 0);
    return g;
}

hipError_t tdc_launch_chain(const TdcDims &d, const tdc_tuning &t, const TdcFusedGeom &g, hipStream_t s,
                            const float *x, const float *uin_p, const float *core_p,
                            const float *uout_p, float *y, const TdcEpi &epi, bool prepare_only)
{
    TdcChainArgs a;
    a.epi = epi;
    a.x = x; a.uin_p = uin_p; a.core_p = core_p; a.uout_p = uout_p; a.y = y;
    a.C = d.C; a.N = d.N; a.H = d.H; a.W = d.W; a.Ho = d.Ho; a.Wo = d.Wo;
    a.K = d.K; a.stride = d.stride; a.pad = d.pad;
    a.NB1 = d.NB1; a.NB3 = d.NB3; a.KG1 = d.KG1;
    a.TH = g.TH; a.TW = g.TW; a.QW = g.QW; a.Q = g.Q; a.P = g.TH * g.TW; a.QB = g.QB; a.PBk = g.PBk;
    a.tiles_x = g.tiles_x;
    a.pitch1 = g.pitch1;
    a.w_core4 = (int)(tdc_packed_floats_core(d) / 4);
    a.w_uout4 = (int)(tdc_packed_floats_uout(d) / 4);
    a.QH = g.QH;
    a.RPR = tdc_runs_per_row(d.W, d.Wo, g.TW, d.K, d.stride, d.pad);
    a.n_sb = (g.QH * a.RPR + 15) / 16;
    a.div_RPR = tdc_make_div((unsigned)a.RPR);
    const int lay = d.nhwc ? TDC_LAY_NHWC : d.s1_runs ? TDC_LAY_NCHW_RUNS : TDC_LAY_NCHW;
    // 16-byte stores of four consecutive pixels need rows of whole quads and a 16-byte aligned y (a slice of a larger
    // tensor may not be); otherwise the same values go out as four 4-byte stores
    a.vec = (g.TW % 4 == 0 && d.Wo % 4 == 0 && ((uintptr_t)y & 15u) == 0) ? 1 : 0;
    a.div_tiles_x = tdc_make_div((unsigned)g.tiles_x); a.div_QW = tdc_make_div((unsigned)g.QW);
    a.tiles = g.tiles_x * g.tiles_y; a.div_tiles = tdc_make_div((unsigned)a.tiles);
    a.xcd_per = a.tiles * d.B / 8; a.xcd_rem = a.tiles * d.B % 8;
    a.div_TW = tdc_make_div((unsigned)g.TW);
    a.inv_mg1 = ((1u << 20) + (unsigned)(d.NB1 / t.mb[0]) - 1u) / (unsigned)(d.NB1 / t.mb[0]);
    dim3 grid((unsigned)(g.tiles_x * g.tiles_y), (unsigned)d.B), block(64 * t.waves[0]);
    switch (t.mb[0]) {
    case 1: return tdc_launch_chain_mb1(a, d.NB2, t.pb[0], g.weights_in_lds, lay, grid, block, g.lds_bytes, s, prepare_only);
    case 2: return tdc_launch_chain_mb2(a, d.NB2, t.pb[0], g.weights_in_lds, lay, grid, block, g.lds_bytes, s, prepare_only);
    case 4: return tdc_launch_chain_mb4(a, d.NB2, t.pb[0], g.weights_in_lds, lay, grid, block, g.lds_bytes, s, prepare_only);
    default: break;
    }
    return hipErrorInvalidValue;
}
