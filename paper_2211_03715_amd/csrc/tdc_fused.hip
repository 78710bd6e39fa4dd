// FUSED variant: one workgroup evaluates all three stages (Eqs. 2, 3, 4) for one
// TH x TW tile of output pixels of one image, and the intermediates never leave the CU.
//
//   stage 1  z1 tile (R1P channels x the QH x QW input tile incl. the K-1 halo) = U_in^T x,
//            x read straight from HBM/L2 into MFMA B operands (each wavefront reads a
//            16-pixel run of one channel row per lane group, contiguous in NCHW), result to LDS.
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
#include "tdc_internal.h"
#include "tdc_mfma.h"

namespace {

struct FusedArgs {
    const float *x, *uin_p, *core_p, *uout_p;
    float *y;
    int C, N, H, W, Ho, Wo, K, stride, pad;
    int NB1, NB2, NB3, KG1;
    int TH, TW, QW, Q, P, QB, PBk;
    int tiles_x;
    int pitch1, pitch2;
};

template <int MB1, int MB2, int MB3, int PB>
__global__ __launch_bounds__(512) void tdc_fused_kernel(FusedArgs a)
{
    extern __shared__ float lds[];
    float *__restrict__ z1s = lds;                              // [16*NB1][pitch1]
    float *__restrict__ z2s = lds + (size_t)16 * a.NB1 * a.pitch1;  // [16*NB2][pitch2]

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const int g = lane >> 4, l16 = lane & 15;
    const int ty = blockIdx.x / a.tiles_x, tx = blockIdx.x - ty * a.tiles_x, b = blockIdx.y;
    const int i0 = ty * a.TH, j0 = tx * a.TW;                   // first output pixel of the tile
    const int h0 = i0 * a.stride - a.pad, w0 = j0 * a.stride - a.pad;  // first input pixel (may be < 0)
    const int HW = a.H * a.W;

    // ------------------------------------------------------------------ stage 1 (Eq. 2)
    {
        const float *__restrict__ xb = a.x + (size_t)b * a.C * HW;
        const int n_pg = (a.QB + PB - 1) / PB, n_mg = (a.NB1 + MB1 - 1) / MB1;
        for (int u = wave; u < n_pg * n_mg; u += nw) {
            const int pg = u % n_pg, mg = u / n_pg;
            const int mvalid = min(MB1, a.NB1 - mg * MB1);
            int xoff[PB];
            bool ok[PB];
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) {
                const int q = 16 * (pg * PB + pb) + l16;
                const int qh = q / a.QW, qw = q - qh * a.QW;
                const int h = h0 + qh, w = w0 + qw;
                ok[pb] = q < a.Q && h >= 0 && h < a.H && w >= 0 && w < a.W;
                xoff[pb] = h * a.W + w;
            }
            tdc_f4 acc[MB1][PB];
#pragma unroll
            for (int mb = 0; mb < MB1; ++mb)
#pragma unroll
                for (int pb = 0; pb < PB; ++pb) acc[mb][pb] = (tdc_f4){0.f, 0.f, 0.f, 0.f};
            for (int kg = 0; kg < a.KG1; ++kg) {
                float bv[PB][4];
#pragma unroll
                for (int pb = 0; pb < PB; ++pb)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int c = 16 * kg + 4 * j + g;
                        bv[pb][j] = (ok[pb] && c < a.C) ? xb[(size_t)c * HW + xoff[pb]] : 0.f;
                    }
                tdc_f4 av[MB1];
#pragma unroll
                for (int mb = 0; mb < MB1; ++mb)
                    av[mb] = (mb < mvalid) ? tdc_load_a4(a.uin_p, mg * MB1 + mb, a.KG1, kg, lane)
                                           : (tdc_f4){0.f, 0.f, 0.f, 0.f};
                tdc_mma_group<MB1, PB>(acc, av, bv, mvalid);
            }
#pragma unroll
            for (int mb = 0; mb < MB1; ++mb)
#pragma unroll
                for (int pb = 0; pb < PB; ++pb)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int row = 16 * (mg * MB1 + mb) + 4 * g + i;
                        const int col = 16 * (pg * PB + pb) + l16;
                        if (mb < mvalid && pg * PB + pb < a.QB) z1s[row * a.pitch1 + col] = acc[mb][pb][i];
                    }
        }
    }
    __syncthreads();

    // ------------------------------------------------------------------ stage 2 (Eq. 3)
    {
        const int n_pg = (a.PBk + PB - 1) / PB, n_mg = (a.NB2 + MB2 - 1) / MB2;
        const int KG2 = a.K * a.K * a.NB1;
        for (int u = wave; u < n_pg * n_mg; u += nw) {
            const int pg = u % n_pg, mg = u / n_pg;
            const int mvalid = min(MB2, a.NB2 - mg * MB2);
            int qbase[PB];
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) {
                const int p = 16 * (pg * PB + pb) + l16;
                const int ph = p / a.TW, pw = p - ph * a.TW;
                qbase[pb] = p < a.P ? ph * a.stride * a.QW + pw * a.stride : 0;
            }
            tdc_f4 acc[MB2][PB];
#pragma unroll
            for (int mb = 0; mb < MB2; ++mb)
#pragma unroll
                for (int pb = 0; pb < PB; ++pb) acc[mb][pb] = (tdc_f4){0.f, 0.f, 0.f, 0.f};
            for (int r = 0; r < a.K; ++r)
                for (int s = 0; s < a.K; ++s) {
                    const int toff = r * a.QW + s;
                    const int kgt = (r * a.K + s) * a.NB1;
                    for (int dg = 0; dg < a.NB1; ++dg) {
                        float bv[PB][4];
#pragma unroll
                        for (int pb = 0; pb < PB; ++pb)
#pragma unroll
                            for (int j = 0; j < 4; ++j)
                                bv[pb][j] = z1s[(16 * dg + 4 * j + g) * a.pitch1 + qbase[pb] + toff];
                        tdc_f4 av[MB2];
#pragma unroll
                        for (int mb = 0; mb < MB2; ++mb)
                            av[mb] = (mb < mvalid) ? tdc_load_a4(a.core_p, mg * MB2 + mb, KG2, kgt + dg, lane)
                                                   : (tdc_f4){0.f, 0.f, 0.f, 0.f};
                        tdc_mma_group<MB2, PB>(acc, av, bv, mvalid);
                    }
                }
#pragma unroll
            for (int mb = 0; mb < MB2; ++mb)
#pragma unroll
                for (int pb = 0; pb < PB; ++pb)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int row = 16 * (mg * MB2 + mb) + 4 * g + i;
                        const int col = 16 * (pg * PB + pb) + l16;
                        if (mb < mvalid && pg * PB + pb < a.PBk) z2s[row * a.pitch2 + col] = acc[mb][pb][i];
                    }
        }
    }
    __syncthreads();

    // ------------------------------------------------------------------ stage 3 (Eq. 4)
    {
        const int n_pg = (a.PBk + PB - 1) / PB, n_mg = (a.NB3 + MB3 - 1) / MB3;
        const int P2 = a.Ho * a.Wo;
        float *__restrict__ yb = a.y + (size_t)b * a.N * P2;
        for (int u = wave; u < n_pg * n_mg; u += nw) {
            const int pg = u % n_pg, mg = u / n_pg;
            const int mvalid = min(MB3, a.NB3 - mg * MB3);
            int yoff[PB];
            bool ok[PB];
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) {
                const int p = 16 * (pg * PB + pb) + l16;
                const int ph = p / a.TW, pw = p - ph * a.TW;
                const int i = i0 + ph, j = j0 + pw;
                ok[pb] = p < a.P && i < a.Ho && j < a.Wo;
                yoff[pb] = i * a.Wo + j;
            }
            tdc_f4 acc[MB3][PB];
#pragma unroll
            for (int mb = 0; mb < MB3; ++mb)
#pragma unroll
                for (int pb = 0; pb < PB; ++pb) acc[mb][pb] = (tdc_f4){0.f, 0.f, 0.f, 0.f};
            for (int kg = 0; kg < a.NB2; ++kg) {
                float bv[PB][4];
#pragma unroll
                for (int pb = 0; pb < PB; ++pb)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int col = min(16 * (pg * PB + pb), 16 * (a.PBk - 1)) + l16;
                        bv[pb][j] = z2s[(16 * kg + 4 * j + g) * a.pitch2 + col];
                    }
                tdc_f4 av[MB3];
#pragma unroll
                for (int mb = 0; mb < MB3; ++mb)
                    av[mb] = (mb < mvalid) ? tdc_load_a4(a.uout_p, mg * MB3 + mb, a.NB2, kg, lane)
                                           : (tdc_f4){0.f, 0.f, 0.f, 0.f};
                tdc_mma_group<MB3, PB>(acc, av, bv, mvalid);
            }
#pragma unroll
            for (int mb = 0; mb < MB3; ++mb)
#pragma unroll
                for (int pb = 0; pb < PB; ++pb)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int n = 16 * (mg * MB3 + mb) + 4 * g + i;
                        if (mb < mvalid && ok[pb] && n < a.N) yb[(size_t)n * P2 + yoff[pb]] = acc[mb][pb][i];
                    }
        }
    }
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
    // smallest pitch >= cols with pitch % 32 == 16: the two 16-lane groups served in one LDS
    // pass (rows k and k+1 of a B operand) then fall into disjoint banks
    int p = (cols + 31) / 32 * 32 + 16;
    if (p - 32 >= cols) p -= 32;
    return p;
}

TdcFusedGeom tdc_fused_geometry(const TdcDims &d, int tile_h, int tile_w)
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
    g.lds_bytes = ((size_t)16 * d.NB1 * g.pitch1 + (size_t)16 * d.NB2 * g.pitch2) * sizeof(float);
    return g;
}

hipError_t tdc_launch_fused(const TdcDims &d, const tdc_tuning &t, const TdcFusedGeom &g, hipStream_t s,
                            const float *x, const float *uin_p, const float *core_p,
                            const float *uout_p, float *y)
{
    FusedArgs a;
    a.x = x; a.uin_p = uin_p; a.core_p = core_p; a.uout_p = uout_p; a.y = y;
    a.C = d.C; a.N = d.N; a.H = d.H; a.W = d.W; a.Ho = d.Ho; a.Wo = d.Wo;
    a.K = d.K; a.stride = d.stride; a.pad = d.pad;
    a.NB1 = d.NB1; a.NB2 = d.NB2; a.NB3 = d.NB3; a.KG1 = d.KG1;
    a.TH = g.TH; a.TW = g.TW; a.QW = g.QW; a.Q = g.Q; a.P = g.TH * g.TW; a.QB = g.QB; a.PBk = g.PBk;
    a.tiles_x = g.tiles_x;
    a.pitch1 = g.pitch1; a.pitch2 = g.pitch2;
    dim3 grid((unsigned)(g.tiles_x * g.tiles_y), (unsigned)d.B), block(64 * t.waves[0]);
#define TDC_X(A_, B_, C_, D_)                                                                          \
    if (t.mb[0] == A_ && t.mb[1] == B_ && t.mb[2] == C_ && t.pb[0] == D_) {                            \
        if (g.lds_bytes > 48 * 1024) {                                                                 \
            hipError_t e = hipFuncSetAttribute((const void *)tdc_fused_kernel<A_, B_, C_, D_>,         \
                                               hipFuncAttributeMaxDynamicSharedMemorySize,             \
                                               (int)g.lds_bytes);                                      \
            if (e != hipSuccess) return e;                                                             \
        }                                                                                              \
        hipLaunchKernelGGL((tdc_fused_kernel<A_, B_, C_, D_>), grid, block, g.lds_bytes, s, a);        \
        return hipGetLastError();                                                                      \
    }
    TDC_FUSED_MENU(TDC_X)
#undef TDC_X
    return hipErrorInvalidValue;
}
