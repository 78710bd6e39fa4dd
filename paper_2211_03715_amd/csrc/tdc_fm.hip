// FUSED_MERGED variant: one launch for the whole layer in the latency regime (batch 1, small ranks).
//
// A workgroup owns one TH x TW tile of output pixels of one image AND one group of NBG 16-channel
// blocks of the output.  It runs
//   stage 1    z1 tile (all R1P channels x the input tile incl. halo) = U_in^T x  (Eq. 2), to LDS,
//              exactly as the FUSED kernel does;
//   stage 2+3  y(n-block, tile) = Wm (*) z1 with Wm = core x_2 U_out (Eqs. 3 and 4 folded into one
//              K x K convolution R1 -> N when the weights were re-laid out), straight to HBM.
// Workgroups that share a tile but own different output-channel groups each recompute stage 1:
// at batch 1 most CUs are idle anyway, and the recomputation buys what the three-stage form cannot
// give on a small image -- parallelism over output channels inside ONE launch, with a single
// barrier between the stages.
//
// Every wavefront owns one output-channel block and one slice of the contraction range
// (k = (tap, d1-block), KG2 = K*K*NB1 k-groups split KS ways; wave = ks*NBG + block), at most FR
// k-groups.  Its FR weight fragments are fetched into registers as the kernel's very first
// instructions, so they travel in the same memory round trip as the first stage-1 operands and
// stage 2+3 touches only LDS (z1 cells) and registers.  Partial sums of the KS slices are added
// through LDS in a fixed order.
#include "tdc_internal.h"
#include "tdc_mfma.h"
#include "tdc_stage1.h"

namespace {

constexpr int FM_FR = 9;     // weight fragments a wavefront may hold (k-groups of its slice)

struct FmArgs {
    const float *x, *uin_p, *wm_p;
    float *y;
    int C, N, H, W, Ho, Wo, K, stride, pad;
    int NB1, NB3, KG1;
    int TH, TW, QW, Q, P, QB;
    int tiles_x, tiles;
    int pitch1;             // LDS row pitch of the z1 tile, in 16-byte cells
    int NBG, KS;            // output-channel blocks per workgroup, contraction slices
    int kg_q, kg_r;         // KG2 = KS * kg_q + kg_r: the first kg_r slices take kg_q + 1 k-groups
    TdcEpi epi;
    TdcDiv div_groups, div_tiles_x, div_NBG, div_QW, div_TW, div_NB1, div_K;   // constant divisors (groups: output-channel groups per tile)
    int n_groups, xcd_per, xcd_rem;   // workgroups per XCD (and the remainder) of the id remap below
    int QH, RPR, n_sb;      // run-major stage 1: tile rows, runs per row, 64-pixel blocks of runs
    TdcDiv div_RPR;
    unsigned inv_mg1;       // ceil(2^20 / (NB1 / mb1)): divides a stage-1 unit index by the channel groups
};

template <int MB1, int PBK, int LAY>
__global__ __launch_bounds__(512) void tdc_fm_kernel(FmArgs a)
{
    constexpr bool NHWC = LAY == TDC_LAY_NHWC;
    extern __shared__ tdc_f4 lds4[];
    tdc_f4 *__restrict__ z1s = lds4;                                   // [NB1][4][pitch1]
    tdc_f4 *__restrict__ red = z1s + (size_t)4 * a.NB1 * a.pitch1;     // [wave][PBK][64]   (KS > 1)

    TDC_PROBE(0);
    unsigned bd = blockDim.x;
    TdcDiv div_groups = a.div_groups;
    TDC_FETCH_NOW(TDC_OUTS("+s"(bd), "+s"(div_groups.m)), "s"(a.x), "s"(a.uin_p), "s"(a.wm_p), "s"(div_groups.sh1), "s"(div_groups.sh2),
                  "s"(a.n_groups), "s"(a.xcd_per), "s"(a.xcd_rem));
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), nw = (int)(bd >> 6);
    const int g = lane >> 4, l16 = lane & 15;
    // Workgroup ids are dealt to the 8 XCDs round-robin, each with its own L2.  Give every XCD one contiguous range of
    // logical ids and make the output-channel group the fast index: the groups of one pixel tile run on one XCD at the
    // same time and pull that tile of x from HBM once instead of once per group.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int lb = xcd * a.xcd_per + min(xcd, a.xcd_rem) + slot;
    const int tile = tdc_div(lb, div_groups), ng = lb - tile * a.n_groups, b = blockIdx.y;
    const int ty = tdc_div(tile, a.div_tiles_x), tx = tile - ty * a.tiles_x;
    const int i0 = ty * a.TH, j0 = tx * a.TW;
    const int h0 = i0 * a.stride - a.pad, w0 = j0 * a.stride - a.pad;
    const int HW = a.H * a.W;
    const int KG2 = a.K * a.K * a.NB1;

    // ---- this wavefront's slice of stage 2+3 and its weight fragments (in flight from here on)
    const int ks = tdc_div(wave, a.div_NBG), nbi = wave - ks * a.NBG;
    const int nb = ng * a.NBG + nbi;
    const int kg0 = ks * a.kg_q + min(ks, a.kg_r), kg1 = kg0 + a.kg_q + (ks < a.kg_r ? 1 : 0);
    tdc_f4 wfrag[FM_FR];

    TDC_PROBE(1);
    // ------------------------------------------------------------------ stage 1 (Eq. 2)
    {
        TdcS1Geom sg;
        sg.x_img = a.x + (size_t)b * a.C * HW; sg.uin_p = a.uin_p;
        sg.C = a.C; sg.H = a.H; sg.W = a.W; sg.KG1 = a.KG1; sg.NB1 = a.NB1;
        sg.QB = a.QB; sg.Q = a.Q; sg.QW = a.QW; sg.h0 = h0; sg.w0 = w0; sg.pitch1 = a.pitch1;
        sg.div_QW = a.div_QW; sg.inv_mg = a.inv_mg1;
        sg.QH = a.QH; sg.RPR = a.RPR; sg.n_sb = a.n_sb; sg.div_RPR = a.div_RPR;
        const auto stage1 = [&](auto &s1) {
            s1.prefetch();
            // The weight fragments of stage 2+3 go out right behind the first stage-1 operands: loads
            // return in order, so stage 1 can start as soon as its own data is there while these are
            // still in flight; a dead fragment (past the slice) reads as zero.
            const tdc_rsrc wrs = tdc_make_rsrc(a.wm_p + (size_t)nb * KG2 * 256, (unsigned)KG2 * 1024u);
#pragma unroll
            for (int f = 0; f < FM_FR; ++f)
                wfrag[f] = tdc_buf_load4(wrs, ((unsigned)(kg0 + f) * 1024u + lane * 16u) | (kg0 + f < kg1 ? 0u : TDC_OOB));
            s1.zero_outside(z1s);
            s1.run(z1s);
        };
        if constexpr (LAY == TDC_LAY_NCHW_RUNS) {
            TdcStage1R<MB1, (MB1 >= 4 ? 1 : 2)> s1(sg, lane, wave, nw);
            stage1(s1);
        } else {
            TdcStage1<MB1, 1, (MB1 >= 4 ? 2 : 4), NHWC> s1(sg, lane, wave, nw);
            stage1(s1);
        }
    }
    TDC_PROBE(2);
    __syncthreads();
    TDC_PROBE(3);

    // ------------------------------------------------------------------ stages 2+3 (Eqs. 3, 4 folded)
    tdc_f4 acc[PBK];
    int qbase[PBK];
#pragma unroll
    for (int pb = 0; pb < PBK; ++pb) {
        acc[pb] = tdc_f4_zero();
        const int p = 16 * pb + l16;
        const int ph = tdc_div(p, a.div_TW), pw = p - ph * a.TW;
        qbase[pb] = g * a.pitch1 + (p < a.P ? ph * a.stride * a.QW + pw * a.stride : 0);
    }
    {
        // position of k-group kg0 within (tap, d1-block); all of it wave-uniform
        const int tap0 = tdc_div(kg0, a.div_NB1);
        int dg = kg0 - tap0 * a.NB1;
        const int r0 = tdc_div(tap0, a.div_K);
        int s = tap0 - r0 * a.K;
        int toff = r0 * a.QW + s;
        // No branch on "fragment f is live": a dead fragment is all zeros and multiplies cell 0, so
        // the LDS reads of all fragments can be issued ahead of the MFMAs.
#pragma unroll
        for (int f = 0; f < FM_FR; ++f) {
            const int cell = kg0 + f < kg1 ? dg * 4 * a.pitch1 + toff : 0;
#pragma unroll
            for (int pb = 0; pb < PBK; ++pb) {
                const tdc_f4 bv = z1s[cell + (kg0 + f < kg1 ? qbase[pb] : 0)];
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[pb] = tdc_mfma(wfrag[f][j], bv[j], acc[pb]);
            }
            const bool wrap_d = ++dg == a.NB1;
            dg = wrap_d ? 0 : dg;
            const bool wrap_s = wrap_d && ++s == a.K;   // s advances only when dg wraps
            toff += wrap_d ? (wrap_s ? a.QW - a.K + 1 : 1) : 0;
            s = wrap_s ? 0 : s;
        }
    }

    TDC_PROBE(4);
    const int P2 = a.Ho * a.Wo;
    float *__restrict__ yb = a.y + (size_t)b * a.N * P2;
    if (a.KS == 1) {
#pragma unroll
        for (int pb = 0; pb < PBK; ++pb) {
            const int p = 16 * pb + l16;
            const int ph = tdc_div(p, a.div_TW), pw = p - ph * a.TW;
            const int i = i0 + ph, j = j0 + pw;
            if (p < a.P && i < a.Ho && j < a.Wo) {
                if (NHWC) {
                    const int n = 16 * nb + 4 * g;
                    if (n < a.N) tdc_store_nhwc(a.y, a.epi, acc[pb], n, ((size_t)b * P2 + i * a.Wo + j) * a.N + n);
                    continue;
                }
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int n = 16 * nb + 4 * g + c;
                    if (n < a.N) {
                        const size_t idx = (size_t)n * P2 + i * a.Wo + j;
                        yb[idx] = tdc_apply_epilogue(a.epi, acc[pb][c], n, (size_t)b * a.N * P2 + idx);
                    }
                }
            }
        }
        TDC_PROBE(7);
        return;
    }
    // partial sums of the KS slices, [wave = ks*NBG + block][pb][lane], then a fixed-order sum
#pragma unroll
    for (int pb = 0; pb < PBK; ++pb) red[(wave * PBK + pb) * 64 + lane] = acc[pb];
    __syncthreads();
    TDC_PROBE(5);
    for (int e = threadIdx.x; e < a.NBG * PBK * 64; e += blockDim.x) {
        const int ln = e & 63, pb = (e >> 6) % PBK, blk = (e >> 6) / PBK;
        tdc_f4 sum = red[(blk * PBK + pb) * 64 + ln];
        for (int k = 1; k < a.KS; ++k) {
            const tdc_f4 v = red[((k * a.NBG + blk) * PBK + pb) * 64 + ln];
            sum += v;
        }
        const int p = 16 * pb + (ln & 15);
        const int ph = tdc_div(p, a.div_TW), pw = p - ph * a.TW;
        const int i = i0 + ph, j = j0 + pw;
        if (p < a.P && i < a.Ho && j < a.Wo) {
            if (NHWC) {
                const int n = 16 * (ng * a.NBG + blk) + 4 * (ln >> 4);
                if (n < a.N) tdc_store_nhwc(a.y, a.epi, sum, n, ((size_t)b * P2 + i * a.Wo + j) * a.N + n);
                continue;
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int n = 16 * (ng * a.NBG + blk) + 4 * (ln >> 4) + c;
                if (n < a.N) {
                    const size_t idx = (size_t)n * P2 + i * a.Wo + j;
                    yb[idx] = tdc_apply_epilogue(a.epi, sum[c], n, (size_t)b * a.N * P2 + idx);
                }
            }
        }
    }
    TDC_PROBE(7);
}

}  // namespace

// nbg = output-channel blocks per workgroup; the workgroup has nw = nbg * KS wavefronts
bool tdc_fm_supported(const TdcDims &d, int tile_h, int tile_w, int nw, int mb1, int nbg)
{
    if (mb1 != 1 && mb1 != 2 && mb1 != 4) return false;
    if (d.NB1 % mb1 || nbg < 1 || d.NB3 % nbg || nw < 1 || nw > 8 || nw % nbg) return false;
    const int pbk = (tile_h * tile_w + 15) / 16;
    if (pbk < 1 || pbk > 4) return false;
    const int ks = nw / nbg, kg2 = d.K * d.K * d.NB1;
    if (ks > kg2) return false;
    return (kg2 + ks - 1) / ks <= FM_FR;   // the longest slice must fit the fragment registers
}

TdcFusedGeom tdc_fm_geometry(const TdcDims &d, int tile_h, int tile_w, int nw, int nbg)
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
    g.weights_in_lds = false;
    g.weights_fit = false;
    const int ks = nbg > 0 ? nw / nbg : 1;
    g.lds_bytes = (size_t)16 * d.NB1 * g.pitch1 * sizeof(float) + (ks > 1 ? (size_t)nw * g.PBk * 1024 : 0);
    return g;
}

hipError_t tdc_launch_fm(const TdcDims &d, const tdc_tuning &t, const TdcFusedGeom &g, hipStream_t s, const float *x,
                         const float *uin_p, const float *wm_p, float *y, const TdcEpi &epi, bool prepare_only)
{
    FmArgs a;
    a.epi = epi;
    a.x = x; a.uin_p = uin_p; a.wm_p = wm_p; a.y = y;
    a.C = d.C; a.N = d.N; a.H = d.H; a.W = d.W; a.Ho = d.Ho; a.Wo = d.Wo;
    a.K = d.K; a.stride = d.stride; a.pad = d.pad;
    a.NB1 = d.NB1; a.NB3 = d.NB3; a.KG1 = d.KG1;
    a.TH = g.TH; a.TW = g.TW; a.QW = g.QW; a.Q = g.Q; a.P = g.TH * g.TW; a.QB = g.QB;
    a.tiles_x = g.tiles_x; a.tiles = g.tiles_x * g.tiles_y;
    a.pitch1 = g.pitch1;
    a.NBG = t.mb[1]; a.KS = t.waves[0] / t.mb[1];
    const int kg2 = d.K * d.K * d.NB1;
    a.kg_q = kg2 / a.KS; a.kg_r = kg2 % a.KS;
    a.n_groups = d.NB3 / a.NBG;
    a.div_groups = tdc_make_div((unsigned)a.n_groups); a.div_tiles_x = tdc_make_div((unsigned)a.tiles_x);
    a.xcd_per = a.tiles * a.n_groups / 8; a.xcd_rem = a.tiles * a.n_groups % 8;
    a.div_NBG = tdc_make_div((unsigned)a.NBG);
    a.inv_mg1 = ((1u << 20) + (unsigned)(d.NB1 / t.mb[0]) - 1u) / (unsigned)(d.NB1 / t.mb[0]);
    a.div_QW = tdc_make_div((unsigned)a.QW); a.div_TW = tdc_make_div((unsigned)a.TW);
    a.div_NB1 = tdc_make_div((unsigned)a.NB1); a.div_K = tdc_make_div((unsigned)a.K);
    a.QH = g.QH;
    a.RPR = tdc_runs_per_row(d.W, d.Wo, g.TW, d.K, d.stride, d.pad);
    a.n_sb = (g.QH * a.RPR + 15) / 16;
    a.div_RPR = tdc_make_div((unsigned)a.RPR);
    const int lay = d.nhwc ? TDC_LAY_NHWC : d.s1_runs ? TDC_LAY_NCHW_RUNS : TDC_LAY_NCHW;
    dim3 grid((unsigned)(a.tiles * (d.NB3 / a.NBG)), (unsigned)d.B), block(64 * t.waves[0]);
#define TDC_FM_LAUNCH(M_, P_, L_)                                                                  \
    {                                                                                              \
        {                                                                                              \
            hipError_t e = tdc_allow_lds((const void *)tdc_fm_kernel<M_, P_, L_>, g.lds_bytes);    \
            if (e != hipSuccess) return e;                                                             \
            if (prepare_only) return hipSuccess;                                                       \
        }                                                                                              \
        hipLaunchKernelGGL((tdc_fm_kernel<M_, P_, L_>), grid, block, g.lds_bytes, s, a);           \
        return hipGetLastError();                                                                  \
    }
#define TDC_FM_CASE(M_, P_)                                                                        \
    if (t.mb[0] == M_ && g.PBk == P_) {                                                            \
        if (lay == TDC_LAY_NHWC) TDC_FM_LAUNCH(M_, P_, TDC_LAY_NHWC)                               \
        else if (lay == TDC_LAY_NCHW_RUNS) TDC_FM_LAUNCH(M_, P_, TDC_LAY_NCHW_RUNS)                \
        else TDC_FM_LAUNCH(M_, P_, TDC_LAY_NCHW)                                                   \
    }
    TDC_FM_CASE(1, 1) TDC_FM_CASE(1, 2) TDC_FM_CASE(1, 3) TDC_FM_CASE(1, 4)
    TDC_FM_CASE(2, 1) TDC_FM_CASE(2, 2) TDC_FM_CASE(2, 3) TDC_FM_CASE(2, 4)
    TDC_FM_CASE(4, 1) TDC_FM_CASE(4, 2) TDC_FM_CASE(4, 3) TDC_FM_CASE(4, 4)
#undef TDC_FM_CASE
#undef TDC_FM_LAUNCH
    return hipErrorInvalidValue;
}
