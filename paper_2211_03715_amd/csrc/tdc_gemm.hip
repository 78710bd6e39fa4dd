// SPLIT variant: the three stages (Eqs. 2, 3, 4) as three fp32-MFMA GEMM kernels,
//   D[b][m][p] = sum_k Wt[k][m] * Act[b][k][p],
// with pixels p along the lanes (contiguous in NCHW), output channels m in the MFMA rows
// and the intermediates z1 [B][R1P][H*W], z2 [B][R2P][Ho*Wo] in plan-owned workspace.
// Stage 2 is an implicit GEMM: k = (tap, d1) and the activation operand is gathered from
// z1 at the tap's offset, with zero for taps that fall outside the image.
//
// One workgroup computes one MB x PB group of 16x16 output blocks.  Its wavefronts split the
// contraction range between them (each takes a contiguous run of 16-wide k-groups) and the
// partial sums are added in a fixed order through LDS, so the result is deterministic.
// Splitting the contraction is what fills the chip on the small-image layers (14x14, 7x7),
// where there are far fewer output blocks than SIMDs; the paper's kernel splits its input
// channels across thread blocks for the same reason (section 5.2) but combines with atomics.
#include "tdc_internal.h"
#include "tdc_mfma.h"

namespace {

struct GemmArgs {
    const float *act;
    const float *wp;
    float *out;
    int act_rows;        // channel rows per image in act (C, R1P, R2P)
    int act_rows_valid;  // rows that exist in memory (C for stage 1, all otherwise)
    int act_pix;         // pixels per row in act
    int out_rows;        // channel rows per image in out (R1P, R2P, N)
    int out_pix;         // pixels per row in out
    int NBm;             // 16-blocks of output channels
    int KG;              // 16-wide k-groups of the contraction
    int NBk;             // stage 2: k-groups per tap (= NB1)
    int n_pgroups;
    int H, W, Wo, K, stride, pad;   // stage 2 geometry
};

template <int MODE, int MB, int PB>
__global__ __launch_bounds__(512) void tdc_gemm_kernel(GemmArgs a)
{
    extern __shared__ float red[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const int g = lane >> 4, l16 = lane & 15;
    const int pg = blockIdx.x % a.n_pgroups, mg = blockIdx.x / a.n_pgroups, b = blockIdx.y;
    const int mvalid = min(MB, a.NBm - mg * MB);

    int poff[PB], ih0[PB], iw0[PB];
    bool pval[PB];
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) {
        const int p = 16 * (pg * PB + pb) + l16;
        pval[pb] = p < a.out_pix;
        if (MODE == 2) {
            const int i = p / a.Wo, j = p - i * a.Wo;
            ih0[pb] = i * a.stride - a.pad;
            iw0[pb] = j * a.stride - a.pad;
            poff[pb] = ih0[pb] * a.W + iw0[pb];
        } else {
            ih0[pb] = iw0[pb] = 0;
            poff[pb] = p;
        }
    }
    const float *__restrict__ actb = a.act + (size_t)b * a.act_rows * a.act_pix;

    tdc_f4 acc[MB][PB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) acc[mb][pb] = (tdc_f4){0.f, 0.f, 0.f, 0.f};

    const int kg0 = (int)(((long)a.KG * wave) / nw), kg1 = (int)(((long)a.KG * (wave + 1)) / nw);
    for (int kg = kg0; kg < kg1; ++kg) {
        float bv[PB][4];
        if (MODE == 2) {
            const int tap = kg / a.NBk, dg = kg - tap * a.NBk;
            const int r = tap / a.K, s = tap - r * a.K;
            const int toff = r * a.W + s;
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) {
                const int h = ih0[pb] + r, w = iw0[pb] + s;
                const bool ok = pval[pb] && h >= 0 && h < a.H && w >= 0 && w < a.W;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int row = 16 * dg + 4 * j + g;
                    bv[pb][j] = ok ? actb[(size_t)row * a.act_pix + poff[pb] + toff] : 0.f;
                }
            }
        } else {
#pragma unroll
            for (int pb = 0; pb < PB; ++pb)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int row = 16 * kg + 4 * j + g;
                    const bool ok = pval[pb] && row < a.act_rows_valid;
                    bv[pb][j] = ok ? actb[(size_t)row * a.act_pix + poff[pb]] : 0.f;
                }
        }
        tdc_f4 av[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            av[mb] = (mb < mvalid) ? tdc_load_a4(a.wp, mg * MB + mb, a.KG, kg, lane) : (tdc_f4){0.f, 0.f, 0.f, 0.f};
        tdc_mma_group<MB, PB>(acc, av, bv, mvalid);
    }

    float *__restrict__ outb = a.out + (size_t)b * a.out_rows * a.out_pix;
    if (nw == 1) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int pb = 0; pb < PB; ++pb)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int m = 16 * (mg * MB + mb) + 4 * g + i;
                    const int p = 16 * (pg * PB + pb) + l16;
                    if (mb < mvalid && m < a.out_rows && p < a.out_pix) outb[(size_t)m * a.out_pix + p] = acc[mb][pb][i];
                }
        return;
    }
    // Partial sums of every wavefront to LDS, [wave][(mb*PB + pb)*4 + i][lane], then a fixed-order sum.
    constexpr int E = MB * PB * 256;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int pb = 0; pb < PB; ++pb)
#pragma unroll
            for (int i = 0; i < 4; ++i) red[wave * E + ((mb * PB + pb) * 4 + i) * 64 + lane] = acc[mb][pb][i];
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += blockDim.x) {
        float sum = red[e];
        for (int w = 1; w < nw; ++w) sum += red[w * E + e];
        const int ln = e & 63, i = (e >> 6) & 3, blk = e >> 8;
        const int pb = blk % PB, mb = blk / PB;
        const int m = 16 * (mg * MB + mb) + 4 * (ln >> 4) + i;
        const int p = 16 * (pg * PB + pb) + (ln & 15);
        if (mb < mvalid && m < a.out_rows && p < a.out_pix) outb[(size_t)m * a.out_pix + p] = sum;
    }
}

template <int MODE>
hipError_t launch_stage(const GemmArgs &a, int mb, int pb, int waves, int batch, hipStream_t s)
{
    const int n_mgroups = (a.NBm + mb - 1) / mb;
    dim3 grid((unsigned)(n_mgroups * a.n_pgroups), (unsigned)batch), block(64 * waves);
    const size_t lds = waves > 1 ? (size_t)waves * mb * pb * 256 * sizeof(float) : 0;
#define TDC_CASE(M_, P_)                                                                          \
    if (mb == M_ && pb == P_) {                                                                   \
        hipLaunchKernelGGL((tdc_gemm_kernel<MODE, M_, P_>), grid, block, lds, s, a);              \
        return hipGetLastError();                                                                 \
    }
    TDC_CASE(1, 1) TDC_CASE(2, 1) TDC_CASE(1, 2) TDC_CASE(2, 2) TDC_CASE(4, 1)
    TDC_CASE(1, 4) TDC_CASE(4, 2) TDC_CASE(2, 4) TDC_CASE(4, 4)
#undef TDC_CASE
    return hipErrorInvalidValue;
}

}  // namespace

bool tdc_gemm_unit_supported(int mb, int pb)
{
    return (mb == 1 || mb == 2 || mb == 4) && (pb == 1 || pb == 2 || pb == 4);
}

hipError_t tdc_launch_split(const TdcDims &d, const tdc_tuning &t, hipStream_t s, const float *x,
                            const float *uin_p, const float *core_p, const float *uout_p,
                            float *z1, float *z2, float *y)
{
    const int HW = d.H * d.W, P = d.Ho * d.Wo;
    GemmArgs a;
    // stage 1 (Eq. 2): z1 = U_in^T x
    a.act = x; a.wp = uin_p; a.out = z1;
    a.act_rows = d.C; a.act_rows_valid = d.C; a.act_pix = HW;
    a.out_rows = 16 * d.NB1; a.out_pix = HW;
    a.NBm = d.NB1; a.KG = d.KG1; a.NBk = 1;
    a.n_pgroups = ((HW + 15) / 16 + t.pb[0] - 1) / t.pb[0];
    a.H = d.H; a.W = d.W; a.Wo = d.Wo; a.K = d.K; a.stride = d.stride; a.pad = d.pad;
    hipError_t e = launch_stage<1>(a, t.mb[0], t.pb[0], t.waves[0], d.B, s);
    if (e != hipSuccess) return e;
    // stage 2 (Eq. 3): z2 = core conv of z1
    a.act = z1; a.wp = core_p; a.out = z2;
    a.act_rows = 16 * d.NB1; a.act_rows_valid = 16 * d.NB1; a.act_pix = HW;
    a.out_rows = 16 * d.NB2; a.out_pix = P;
    a.NBm = d.NB2; a.KG = d.K * d.K * d.NB1; a.NBk = d.NB1;
    a.n_pgroups = ((P + 15) / 16 + t.pb[1] - 1) / t.pb[1];
    e = launch_stage<2>(a, t.mb[1], t.pb[1], t.waves[1], d.B, s);
    if (e != hipSuccess) return e;
    // stage 3 (Eq. 4): y = U_out^T z2
    a.act = z2; a.wp = uout_p; a.out = y;
    a.act_rows = 16 * d.NB2; a.act_rows_valid = 16 * d.NB2; a.act_pix = P;
    a.out_rows = d.N; a.out_pix = P;
    a.NBm = d.NB3; a.KG = d.NB2; a.NBk = 1;
    a.n_pgroups = ((P + 15) / 16 + t.pb[2] - 1) / t.pb[2];
    return launch_stage<3>(a, t.mb[2], t.pb[2], t.waves[2], d.B, s);
}
