// FUSED variant: one workgroup evaluates all three stages (Eqs. 2, 3, 4) for one
// TH x TW tile of output pixels of one image, and the intermediates never leave the CU.
//
//   stage 1  z1 tile (R1P channels x the QH x QW input tile incl. the K-1 halo) = U_in^T x,
//            x read straight from HBM/L2 into MFMA B operands (NCHW: each wavefront reads a
//            16-pixel run of one channel row per lane group with 4-byte loads; NHWC, template
//            flag: a lane's four channels of its pixel are one 16-byte load), result to LDS.
//            Pixels of the halo that lie outside the image read x = 0, which is the zero
//            padding of the core convolution because stage 1 has no bias.
//   stage 2  z2 tile (R2P x TH*TW) = core conv, an implicit GEMM over k = (tap, d1) whose B
//            operands are ds_reads of the z1 tile at the tap's offset; accumulators in
//            registers, result to LDS.
//   stage 3  y tile (N x TH*TW) = U_out^T z2, B operands from LDS, result to HBM.
//
// This keeps the idea the paper's core kernel is built on -- the R1-channel input tile and
// its halo stay in on-chip memory while every output channel consumes them (section 5.2) --
// but the lanes run over pixels rather than output channels (64-wide wavefronts, ranks as
// small as 16), the output channels sit in MFMA accumulator registers, nothing is combined
// with atomics, and the two 1x1 stages ride in the same launch.
//
// Each stage's 16x16 output blocks are grouped into MB x PB register tiles ("units") and the
// units are dealt round-robin to the wavefronts of the workgroup.
//
// Latency discipline (a batch-1 layer is a few hundred MFMAs per wavefront, so memory round
// trips, not arithmetic, set the time): every wavefront first issues the loads of its first
// stage-1 tile (x and U_in, straight from global memory), then the workgroup copies the core
// and U_out weights into LDS while those loads are in flight (template flag WLDS; when the
// weights do not fit, stages 2 and 3 stream them from L2 through the same register pipeline).
// After that, stages 2 and 3 touch only LDS.
#include <type_traits>

#include "tdc_internal.h"
#include "tdc_mfma.h"
#include "tdc_stage1.h"

namespace {

struct FusedArgs {
    const float *x, *uin_p, *core_p, *uout_p;
    float *y;
    int C, N, H, W, Ho, Wo, K, stride, pad;
    int NB1, NB2, NB3, KG1;
    int TH, TW, QW, Q, P, QB, PBk;
    int tiles_x;
    int pitch1, pitch2;     // LDS row pitches of the z1 / z2 tiles, in 16-byte units
    int w_core4, w_uout4;   // 16-byte units of the packed core / U_out arrays
    int QH, RPR, n_sb;      // run-major stage 1: tile rows, runs per row, 64-pixel blocks of runs
    TdcDiv div_RPR;
    TdcEpi epi;
    TdcDiv div_tiles_x, div_QW, div_TW, div_npg2, div_tiles;   // launch-time constant divisors (npg2: pixel groups of stages 2, 3)
    int tiles, xcd_per, xcd_rem;   // tiles per image; workgroups per XCD (and the remainder) of the id remap
    unsigned inv_mg1;       // ceil(2^20 / (NB1 / mb1)): divides a stage-1 unit index by the channel groups
};

// LDS tiles hold 16-byte cells: cell (cb, g, col) = channels 16*cb + 4*g + {0,1,2,3} of pixel col,
// i.e. exactly the four accumulator registers of lane (g, col%16) for channel block cb, and
// exactly the B operand of the next stage for k-group cb (see tdc_mfma.h).
__device__ __forceinline__ int tdc_cell(int cb, int g, int pitch, int col) { return (cb * 4 + g) * pitch + col; }

template <int MB1, int MB2, int MB3, int PB, bool WLDS, int LAY>
__global__ __launch_bounds__(512) void tdc_fused_kernel(FusedArgs a)
{
    constexpr bool NHWC = LAY == TDC_LAY_NHWC;
    extern __shared__ tdc_f4 lds4[];
    tdc_f4 *__restrict__ z1s = lds4;                                  // [NB1][4][pitch1]
    tdc_f4 *__restrict__ z2s = z1s + (size_t)4 * a.NB1 * a.pitch1;    // [NB2][4][pitch2]
    tdc_f4 *__restrict__ wC = z2s + (size_t)4 * a.NB2 * a.pitch2;     // packed core   (WLDS)
    tdc_f4 *__restrict__ wO = wC + a.w_core4;                         // packed U_out  (WLDS)

    // every argument stage 1 needs, in one round of scalar loads (see TDC_FETCH_NOW)
    unsigned bd = blockDim.x;
    TdcDiv div_tiles_x = a.div_tiles_x;
    TDC_FETCH_NOW(TDC_OUTS("+s"(bd), "+s"(div_tiles_x.m)), "s"(a.x), "s"(a.uin_p), "s"(a.core_p), "s"(a.uout_p), "s"(a.y), "s"(a.C), "s"(a.H), "s"(a.W),
                  "s"(a.stride), "s"(a.pad), "s"(a.NB1), "s"(a.KG1), "s"(a.TH), "s"(a.TW), "s"(a.QW), "s"(a.Q), "s"(a.QB), "s"(a.tiles_x),
                  "s"(a.pitch1), "s"(a.w_core4), "s"(a.w_uout4), "s"(a.QH), "s"(a.RPR), "s"(a.n_sb), "s"(a.div_RPR.m), "s"(a.div_RPR.sh1),
                  "s"(a.div_RPR.sh2), "s"(div_tiles_x.sh1), "s"(div_tiles_x.sh2),
                  "s"(a.div_QW.m), "s"(a.div_QW.sh1), "s"(a.div_QW.sh2), "s"(a.inv_mg1), "s"(a.tiles), "s"(a.xcd_per), "s"(a.xcd_rem),
                  "s"(a.div_tiles.m), "s"(a.div_tiles.sh1), "s"(a.div_tiles.sh2));
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), nw = (int)(bd >> 6);
    const int g = lane >> 4, l16 = lane & 15;
    // Workgroups are dealt to the 8 XCDs round-robin in launch order (x fastest), each XCD with its own L2.  Every
    // XCD gets one contiguous range of (image, tile) pairs instead, so the tiles that share halo rows and columns of x
    // run on one XCD at the same time and those pixels come from HBM once.
    const int lin = blockIdx.y * a.tiles + blockIdx.x;
    const int xcd = lin & 7, slot = lin >> 3;
    const int lb = xcd * a.xcd_per + min(xcd, a.xcd_rem) + slot;
    const int b = tdc_div(lb, a.div_tiles), tile = lb - b * a.tiles;
    const int ty = tdc_div(tile, div_tiles_x), tx = tile - ty * a.tiles_x;
    const int i0 = ty * a.TH, j0 = tx * a.TW;                   // first output pixel of the tile
    const int h0 = i0 * a.stride - a.pad, w0 = j0 * a.stride - a.pad;  // first input pixel (may be < 0)
    const int HW = a.H * a.W;

    TDC_PROBE(0);
    // ------------------------------------------------------------------ stage 1 (Eq. 2)
    {
        TdcS1Geom sg;
        sg.x_img = a.x + (size_t)b * a.C * HW; sg.uin_p = a.uin_p;
        sg.C = a.C; sg.H = a.H; sg.W = a.W; sg.KG1 = a.KG1; sg.NB1 = a.NB1;
        sg.QB = a.QB; sg.Q = a.Q; sg.QW = a.QW; sg.h0 = h0; sg.w0 = w0; sg.pitch1 = a.pitch1;
        sg.div_QW = a.div_QW; sg.inv_mg = a.inv_mg1;
        sg.QH = a.QH; sg.RPR = a.RPR; sg.n_sb = a.n_sb; sg.div_RPR = a.div_RPR;
        const tdc_f4 *__restrict__ core4 = reinterpret_cast<const tdc_f4 *>(a.core_p);
        const tdc_f4 *__restrict__ uout4 = reinterpret_cast<const tdc_f4 *>(a.uout_p);
        const auto stage1 = [&](auto &s1) {
            s1.prefetch();
            TDC_PROBE(1);
            // core and U_out -> LDS: the first round's loads are issued here, behind the first stage-1
            // operands, and stored after stage 1
            TdcWeightCopy<8> wc;
            if (WLDS) wc.load(core4, a.w_core4, uout4, a.w_uout4, 0);
            TDC_PROBE(2);
            s1.zero_outside(z1s);
            s1.run(z1s);
            if (WLDS) {
                const int n = a.w_core4 + a.w_uout4, round = 8 * (int)blockDim.x;
                wc.store(wC, n, 0);
                for (int base = round; base < n; base += round) {
                    wc.load(core4, a.w_core4, uout4, a.w_uout4, base);
                    wc.store(wC, n, base);
                }
            }
        };
        if constexpr (LAY == TDC_LAY_NCHW_RUNS) {
            TdcStage1R<MB1, (MB1 >= 4 ? 1 : 2)> s1(sg, lane, wave, nw);
            stage1(s1);
        } else {
            TdcStage1<MB1, PB, (MB1 * PB >= 8 ? 2 : 4), NHWC> s1(sg, lane, wave, nw);   // k-groups per operand buffer
            stage1(s1);
        }
    }
    TDC_PROBE(3);
    __syncthreads();
    TDC_PROBE(4);

    // ------------------------------------------------------------------ stage 2 (Eq. 3)
    {
        constexpr int U = WLDS ? 1 : 4;
        const int n_pg = (a.PBk + PB - 1) / PB, n_mg = a.NB2 / MB2;
        const int KG2 = a.K * a.K * a.NB1;
        const tdc_rsrc wrs = tdc_make_rsrc(a.core_p, (unsigned)a.w_core4 * 16u);
        for (int u = wave; u < n_pg * n_mg; u += nw) {
            const int mg = tdc_div(u, a.div_npg2), pg = u - mg * n_pg;
            int qbase[PB];
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) {
                const int p = 16 * (pg * PB + pb) + l16;
                const int ph = tdc_div(p, a.div_TW), pw = p - ph * a.TW;
                qbase[pb] = g * a.pitch1 + (p < a.P ? ph * a.stride * a.QW + pw * a.stride : 0);
            }
            int kg = 0, dg = 0, s = 0, toff = 0;     // toff = r*QW + s
            auto next = [&](tdc_f4(&av)[MB2], tdc_f4(&bv)[PB]) {
                const bool live = kg < KG2;
#pragma unroll
                for (int mb = 0; mb < MB2; ++mb) {
                    const int frag = (mg * MB2 + mb) * KG2 + kg;
                    // WLDS: a dead fetch is never multiplied (one k-group per buffer), it only has to stay in range
                    if (WLDS) av[mb] = wC[(live ? frag : 0) * 64 + lane];
                    else av[mb] = tdc_buf_load4(wrs, ((unsigned)frag * 1024u + lane * 16u) | (live ? 0u : TDC_OOB));
                }
                const int cell = live ? dg * 4 * a.pitch1 + toff : 0;
#pragma unroll
                for (int pb = 0; pb < PB; ++pb) bv[pb] = z1s[cell + qbase[pb]];
                ++kg;
                if (++dg == a.NB1) {
                    dg = 0;
                    ++toff;
                    if (++s == a.K) {
                        s = 0;
                        toff += a.QW - a.K;
                    }
                }
            };
            TdcPipe<MB2, PB, U> pipe;
            tdc_f4 acc[MB2][PB];
            TDC_PROBE(8);
            pipe.start(next);
            pipe.run(acc, KG2, next);
            TDC_PROBE(9);
#pragma unroll
            for (int mb = 0; mb < MB2; ++mb)
#pragma unroll
                for (int pb = 0; pb < PB; ++pb)
                    if (pg * PB + pb < a.PBk)
                        z2s[tdc_cell(mg * MB2 + mb, g, a.pitch2, 16 * (pg * PB + pb) + l16)] = acc[mb][pb];
        }
    }
    TDC_PROBE(5);
    __syncthreads();
    TDC_PROBE(6);

    // ------------------------------------------------------------------ stage 3 (Eq. 4)
    {
        constexpr int U = WLDS ? 1 : 4;
        const int n_pg = (a.PBk + PB - 1) / PB, n_mg = a.NB3 / MB3;
        const int P2 = a.Ho * a.Wo;
        float *__restrict__ yb = a.y + (size_t)b * a.N * P2;
        const tdc_rsrc wrs = tdc_make_rsrc(a.uout_p, (unsigned)a.w_uout4 * 16u);
        // The loop over register tiles exists twice, with and without the epilogue: the epilogue's loads (bias,
        // shortcut) would put waits on the vector-memory counter into it, and that counter also holds the y stores
        // of the previous tile.  The plain loop stores and moves on.
        const auto stage3 = [&](auto with_epi) {
            constexpr bool EPI = decltype(with_epi)::value;
            for (int u = wave; u < n_pg * n_mg; u += nw) {
                const int mg = tdc_div(u, a.div_npg2), pg = u - mg * n_pg;
                int yoff[PB], col[PB];
                bool ok[PB];
#pragma unroll
                for (int pb = 0; pb < PB; ++pb) {
                    const int p = 16 * (pg * PB + pb) + l16;
                    const int ph = tdc_div(p, a.div_TW), pw = p - ph * a.TW;
                    const int i = i0 + ph, j = j0 + pw;
                    ok[pb] = p < a.P && i < a.Ho && j < a.Wo;
                    yoff[pb] = i * a.Wo + j;
                    col[pb] = g * a.pitch2 + min(16 * (pg * PB + pb), 16 * (a.PBk - 1)) + l16;
                }
                int kg = 0;
                auto next = [&](tdc_f4(&av)[MB3], tdc_f4(&bv)[PB]) {
                    const bool live = kg < a.NB2;
                    const int kgc = live ? kg : 0;
#pragma unroll
                    for (int mb = 0; mb < MB3; ++mb) {
                        const int frag = (mg * MB3 + mb) * a.NB2 + kg;
                        if (WLDS) av[mb] = wO[(live ? frag : 0) * 64 + lane];
                        else av[mb] = tdc_buf_load4(wrs, ((unsigned)frag * 1024u + lane * 16u) | (live ? 0u : TDC_OOB));
                    }
#pragma unroll
                    for (int pb = 0; pb < PB; ++pb) bv[pb] = z2s[kgc * 4 * a.pitch2 + col[pb]];
                    ++kg;
                };
                TdcPipe<MB3, PB, U> pipe;
                tdc_f4 acc[MB3][PB];
                pipe.start(next);
                pipe.run(acc, a.NB2, next);
#pragma unroll
                for (int mb = 0; mb < MB3; ++mb)
#pragma unroll
                    for (int pb = 0; pb < PB; ++pb) {
                        if (NHWC) {
                            const int n = 16 * (mg * MB3 + mb) + 4 * g;
                            if (ok[pb] && n < a.N) {
                                const size_t cell = ((size_t)b * P2 + yoff[pb]) * a.N + n;
                                if constexpr (EPI) tdc_store_nhwc(a.y, a.epi, acc[mb][pb], n, cell);
                                else *reinterpret_cast<tdc_f4 *>(a.y + cell) = acc[mb][pb];
                            }
                            continue;
                        }
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int n = 16 * (mg * MB3 + mb) + 4 * g + i;
                            if (ok[pb] && n < a.N) {
                                const size_t idx = (size_t)n * P2 + yoff[pb];
                                if constexpr (EPI) yb[idx] = tdc_apply_epilogue(a.epi, acc[mb][pb][i], n, (size_t)b * a.N * P2 + idx);
                                else yb[idx] = acc[mb][pb][i];
                            }
                        }
                    }
            }
        };
        if (a.epi.bias || a.epi.residual || a.epi.relu) stage3(std::true_type{});
        else stage3(std::false_type{});
    }
    TDC_PROBE(7);
}

#define TDC_FUSED_MENU(X) X(1, 1, 1, 1) X(1, 1, 2, 1) X(2, 2, 2, 1) X(2, 2, 4, 1) X(4, 4, 4, 1) \
                          X(1, 1, 2, 2) X(2, 2, 2, 2) X(2, 2, 4, 2) X(4, 4, 4, 2) X(1, 1, 1, 2)

}  // namespace

bool tdc_fused_unit_supported(int mb1, int mb2, int mb3, int pb)
{
#define TDC_X(A_, B_, C_, D_) if (mb1 == A_ && mb2 == B_ && mb3 == C_ && pb == D_) return true;
    TDC_FUSED_MENU(TDC_X)
#undef TDC_X
    return false;
}

static int round_pitch(int cols)
{
    // row pitch of an LDS tile in 16-byte cells: the columns plus 4 cells (64 bytes), so that
    // the four lane groups of one access start in different banks
    return cols + 4;
}

TdcFusedGeom tdc_fused_geometry(const TdcDims &d, int tile_h, int tile_w, int lds_limit)
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
    g.pitch1 = round_pitch(16 * g.QB);
    g.pitch2 = round_pitch(16 * g.PBk);
    const size_t tiles = ((size_t)16 * d.NB1 * g.pitch1 + (size_t)16 * d.NB2 * g.pitch2) * sizeof(float);
    const size_t weights = (tdc_packed_floats_core(d) + tdc_packed_floats_uout(d)) * sizeof(float);
    g.weights_in_lds = tiles + weights <= (size_t)lds_limit;
    g.weights_fit = g.weights_in_lds;
    g.lds_bytes = tiles + (g.weights_in_lds ? weights : 0);
    return g;
}

hipError_t tdc_launch_fused(const TdcDims &d, const tdc_tuning &t, const TdcFusedGeom &g, hipStream_t s,
                            const float *x, const float *uin_p, const float *core_p,
                            const float *uout_p, float *y, const TdcEpi &epi, bool prepare_only)
{
    FusedArgs a;
    a.epi = epi;
    a.x = x; a.uin_p = uin_p; a.core_p = core_p; a.uout_p = uout_p; a.y = y;
    a.C = d.C; a.N = d.N; a.H = d.H; a.W = d.W; a.Ho = d.Ho; a.Wo = d.Wo;
    a.K = d.K; a.stride = d.stride; a.pad = d.pad;
    a.NB1 = d.NB1; a.NB2 = d.NB2; a.NB3 = d.NB3; a.KG1 = d.KG1;
    a.TH = g.TH; a.TW = g.TW; a.QW = g.QW; a.Q = g.Q; a.P = g.TH * g.TW; a.QB = g.QB; a.PBk = g.PBk;
    a.tiles_x = g.tiles_x;
    a.pitch1 = g.pitch1; a.pitch2 = g.pitch2;
    a.w_core4 = (int)(tdc_packed_floats_core(d) / 4);
    a.w_uout4 = (int)(tdc_packed_floats_uout(d) / 4);
    a.div_tiles_x = tdc_make_div((unsigned)g.tiles_x); a.div_QW = tdc_make_div((unsigned)g.QW);
    a.div_TW = tdc_make_div((unsigned)g.TW);
    a.tiles = g.tiles_x * g.tiles_y; a.div_tiles = tdc_make_div((unsigned)a.tiles);
    a.xcd_per = a.tiles * d.B / 8; a.xcd_rem = a.tiles * d.B % 8;
    a.inv_mg1 = ((1u << 20) + (unsigned)(d.NB1 / t.mb[0]) - 1u) / (unsigned)(d.NB1 / t.mb[0]);
    a.div_npg2 = tdc_make_div((unsigned)((g.PBk + t.pb[0] - 1) / t.pb[0]));
    a.QH = g.QH;
    a.RPR = tdc_runs_per_row(d.W, d.Wo, g.TW, d.K, d.stride, d.pad);
    a.n_sb = (g.QH * a.RPR + 15) / 16;
    a.div_RPR = tdc_make_div((unsigned)a.RPR);
    const int lay = d.nhwc ? TDC_LAY_NHWC : d.s1_runs ? TDC_LAY_NCHW_RUNS : TDC_LAY_NCHW;
    dim3 grid((unsigned)(g.tiles_x * g.tiles_y), (unsigned)d.B), block(64 * t.waves[0]);
#define TDC_LAUNCH(A_, B_, C_, D_, W_, L_)                                                             \
    {                                                                                                  \
        {                                                                                              \
            hipError_t e = tdc_allow_lds((const void *)tdc_fused_kernel<A_, B_, C_, D_, W_, L_>, g.lds_bytes);    \
            if (e != hipSuccess) return e;                                                             \
            if (prepare_only) return hipSuccess;                                                       \
        }                                                                                              \
        hipLaunchKernelGGL((tdc_fused_kernel<A_, B_, C_, D_, W_, L_>), grid, block, g.lds_bytes, s, a);\
        return hipGetLastError();                                                                      \
    }
#define TDC_X(A_, B_, C_, D_)                                                                          \
    if (t.mb[0] == A_ && t.mb[1] == B_ && t.mb[2] == C_ && t.pb[0] == D_) {                            \
        if (g.weights_in_lds) {                                                                        \
            if (lay == TDC_LAY_NHWC) TDC_LAUNCH(A_, B_, C_, D_, true, TDC_LAY_NHWC)                    \
            else if (lay == TDC_LAY_NCHW_RUNS) TDC_LAUNCH(A_, B_, C_, D_, true, TDC_LAY_NCHW_RUNS)     \
            else TDC_LAUNCH(A_, B_, C_, D_, true, TDC_LAY_NCHW)                                        \
        } else {                                                                                       \
            if (lay == TDC_LAY_NHWC) TDC_LAUNCH(A_, B_, C_, D_, false, TDC_LAY_NHWC)                   \
            else if (lay == TDC_LAY_NCHW_RUNS) TDC_LAUNCH(A_, B_, C_, D_, false, TDC_LAY_NCHW_RUNS)    \
            else TDC_LAUNCH(A_, B_, C_, D_, false, TDC_LAY_NCHW)                                       \
        }                                                                                              \
    }
    TDC_FUSED_MENU(TDC_X)
#undef TDC_X
#undef TDC_LAUNCH
    return hipErrorInvalidValue;
}
