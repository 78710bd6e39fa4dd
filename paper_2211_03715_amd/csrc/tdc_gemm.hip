// SPLIT variant: the three stages (Eqs. 2, 3, 4) as three fp32-MFMA GEMM kernels,
//   D[b][m][p] = sum_k Wt[k][m] * Act[b][k][p],
// with pixels p along the lanes, output channels m in the MFMA rows
// and the intermediates z1, z2 in plan-owned workspace in a blocked layout,
//   z[b][channel block cb][pixel][16 channels],
// which is the accumulator layout of the producing kernel (a lane holds channels 4g..4g+3 of one
// pixel: one 16-byte store) and the B-operand layout of the consuming one (one 16-byte load per
// lane and k-group, a wavefront reading 16 pixels x 64 bytes): the intermediates never pay the
// four 4-byte loads per k-group that NCHW activations cost.
// Stage 2 is an implicit GEMM: k = (tap, d1) and the activation operand is gathered from
// z1 at the tap's offset, with zero for taps that fall outside the image.
//
// One workgroup computes one MB x PB group of 16x16 output blocks.  Its wavefronts split the
// contraction range between them (each takes a contiguous run of 16-wide k-groups) and the
// partial sums are added in a fixed order through LDS, so the result is deterministic.
// Splitting the contraction is what fills the chip on the small-image layers (14x14, 7x7),
// where there are far fewer output blocks than SIMDs; the paper's kernel splits its input
// channels across thread blocks for the same reason (section 5.2) but combines with atomics.
//
// At batch 1 a wavefront has only a handful of k-groups, so the kernel is bound by memory
// latency, not by MFMA issue.  The inner loop is therefore branch-free (buffer loads whose
// range check zeroes dead operands) and software-pipelined: operands are fetched U k-groups
// at a time into two register buffers (TdcPipe), U chosen on the host so that 2*U covers the
// wavefront's k-groups whenever they are at most eight -- one memory round trip per kernel.
#include <algorithm>

#include "tdc_internal.h"
#include "tdc_mfma.h"

namespace {

struct GemmArgs {
    const float *act;
    const float *wp;
    float *out;
    int act_rows;        // channel rows per image in act (C, R1P, R2P)
    int act_rows_valid;  // rows that exist in memory (C for stage 1, all otherwise)
    int out_layout;      // TDC_ACT_BLOCKED: an intermediate (see the head of this file); else the layer's y, NCHW or NHWC
    TdcEpi epi;          // applied to the layer's y only
    int act_pix;         // pixels per row in act
    int out_rows;        // channel rows per image in out (R1P, R2P, N)
    int out_pix;         // pixels per row in out
    int NBm;             // 16-blocks of output channels (a multiple of MB)
    int KG;              // 16-wide k-groups of the contraction
    int NBk;             // stage 2: k-groups per tap (= NB1)
    int n_pgroups, n_mgroups;
    int pg_major;        // order of the logical workgroup ids, see tdc_logical_block
    int H, W, Wo, K, stride, pad;   // stage 2 geometry
    int kg_q, kg_r;      // KG = waves * kg_q + kg_r: the first kg_r wavefronts take kg_q + 1 k-groups
    TdcDiv div_inner, div_Wo, div_NBk, div_K;   // launch-time constant divisors (see tdc_div.h)
};

// Workgroups are dealt to the chip's 8 XCDs round-robin by blockIdx.x, and every XCD has its own
// L2.  Remap so that each XCD gets one contiguous range of logical ids: neighbours in the logical
// order -- workgroups that share a weight block (channel-group-major order) or an activation
// block (pixel-group-major order) -- then fetch that operand into one L2 instead of eight.
__device__ __forceinline__ int tdc_logical_block(int bid, int n)
{
    constexpr int XCDS = 8;
    const int per = n / XCDS, rem = n % XCDS;
    const int xcd = bid % XCDS, slot = bid / XCDS;
    return xcd * per + min(xcd, rem) + slot;
}

// Stateful operand fetcher of one wavefront: each call returns the next k-group of its range.
// ACT: layout of the activation operand -- the caller's x (NCHW: four 4-byte loads per lane and
// k-group, one per channel row; NHWC: the lane's four channels are 16 contiguous bytes) or a
// blocked intermediate.
template <int MODE, int ACT, int MB, int PB>
struct GemmNext {
    tdc_rsrc wrs, ars;                // packed weights of this tile's first m-block; activations of this image
    unsigned wlane;                   // byte offset of this lane inside a 1 KiB weight fragment
    unsigned wstride;                 // bytes between consecutive m-blocks (KG fragments)
    int act_pix;
    int C;                            // NHWC: channels per pixel (rows that exist)
    int kg, kg_end;                   // next k-group, end of range (wave-uniform)
    int dg, r, s, NBk, K, H, W;       // stage 2: position of kg within (tap, d1-group)
    int g;
    int poff[PB], ih0[PB], iw0[PB];
    bool pval[PB];

    __device__ __forceinline__ void operator()(tdc_f4 (&av)[MB], tdc_f4 (&bv)[PB])
    {
        const unsigned dead = kg < kg_end ? 0u : TDC_OOB;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) av[mb] = tdc_buf_load4(wrs, (mb * wstride + (unsigned)kg * 1024u + wlane) | dead);
        if (MODE == 2) {
            const int toff = r * W + s;
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) {
                const int h = ih0[pb] + r, w = iw0[pb] + s;
                const bool ok = pval[pb] && h >= 0 && h < H && w >= 0 && w < W;
                const unsigned bad = ok ? dead : TDC_OOB;
                if (ACT == TDC_ACT_BLOCKED) {
                    bv[pb] = tdc_buf_load4(ars, ((unsigned)((dg * act_pix + poff[pb] + toff) * 16 + 4 * g) * 4u) | bad);
                } else if (ACT == TDC_ACT_NHWC) {
                    const int c = 16 * dg + 4 * g;
                    bv[pb] = tdc_buf_load4(ars, ((unsigned)((poff[pb] + toff) * C + c) * 4u) | bad | (c < C ? 0u : TDC_OOB));
                } else {
                    const unsigned base = (unsigned)((16 * dg + 4 * g) * act_pix + poff[pb] + toff) * 4u;
                    bv[pb] = (tdc_f4){tdc_buf_load(ars, base | bad), tdc_buf_load(ars, (base + 4u * act_pix) | bad),
                                      tdc_buf_load(ars, (base + 8u * act_pix) | bad),
                                      tdc_buf_load(ars, (base + 12u * act_pix) | bad)};
                }
            }
            if (++dg == NBk) {
                dg = 0;
                if (++s == K) {
                    s = 0;
                    ++r;
                }
            }
        } else {
            // NCHW: rows past the last channel lie beyond the descriptor and read as 0 by themselves
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) {
                const unsigned bad = pval[pb] ? dead : TDC_OOB;
                if (ACT == TDC_ACT_BLOCKED) {
                    bv[pb] = tdc_buf_load4(ars, ((unsigned)((kg * act_pix + poff[pb]) * 16 + 4 * g) * 4u) | bad);
                } else if (ACT == TDC_ACT_NHWC) {
                    const int c = 16 * kg + 4 * g;
                    bv[pb] = tdc_buf_load4(ars, ((unsigned)(poff[pb] * C + c) * 4u) | bad | (c < C ? 0u : TDC_OOB));
                } else {
                    const unsigned base = (unsigned)((16 * kg + 4 * g) * act_pix + poff[pb]) * 4u;
                    bv[pb] = (tdc_f4){tdc_buf_load(ars, base | bad), tdc_buf_load(ars, (base + 4u * act_pix) | bad),
                                      tdc_buf_load(ars, (base + 8u * act_pix) | bad),
                                      tdc_buf_load(ars, (base + 12u * act_pix) | bad)};
                }
            }
        }
        ++kg;
    }
};

template <int MODE, int ACT, int MB, int PB, int U>
__global__ __launch_bounds__(512) void tdc_gemm_kernel(GemmArgs a)
{
    extern __shared__ float red[];
    unsigned bd = blockDim.x, gd = gridDim.x;
    TdcDiv div_inner = a.div_inner;
    TDC_FETCH_NOW(TDC_OUTS("+s"(bd), "+s"(gd), "+s"(div_inner.m)), "s"(a.act), "s"(a.wp), "s"(a.out), "s"(a.act_rows),
                  "s"(a.act_rows_valid), "s"(a.out_layout), "s"(a.act_pix), "s"(a.out_pix), "s"(a.KG), "s"(a.NBk), "s"(a.n_pgroups),
                  "s"(a.n_mgroups), "s"(a.pg_major), "s"(a.kg_q), "s"(a.kg_r), "s"(div_inner.sh1), "s"(div_inner.sh2), "s"(a.div_Wo.m),
                  "s"(a.div_Wo.sh1), "s"(a.div_Wo.sh2), "s"(a.H), "s"(a.W), "s"(a.Wo), "s"(a.stride), "s"(a.pad));
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), nw = (int)(bd >> 6);
    const int g = lane >> 4, l16 = lane & 15;
    const int lb = tdc_logical_block(blockIdx.x, (int)gd);
    const int inner = a.pg_major ? a.n_mgroups : a.n_pgroups;   // one division on the way to the first load
    const int hi = tdc_div(lb, div_inner), lo = lb - hi * inner;
    const int pg = a.pg_major ? hi : lo, mg = a.pg_major ? lo : hi;
    const int b = blockIdx.y;

    GemmNext<MODE, ACT, MB, PB> next;
    next.wstride = (unsigned)a.KG * 1024u;
    next.wrs = tdc_make_rsrc(a.wp + (size_t)mg * MB * a.KG * 256, MB * next.wstride);
    next.ars = tdc_make_rsrc(a.act + (size_t)b * a.act_rows * a.act_pix, (unsigned)a.act_rows_valid * a.act_pix * 4u);
    next.wlane = lane * 16u;
    next.act_pix = a.act_pix;
    next.C = a.act_rows_valid;
    next.NBk = a.NBk; next.K = a.K; next.H = a.H; next.W = a.W; next.g = g;
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) {
        const int p = 16 * (pg * PB + pb) + l16;
        next.pval[pb] = p < a.out_pix;
        if (MODE == 2) {
            const int i = tdc_div(p, a.div_Wo), j = p - i * a.Wo;
            next.ih0[pb] = i * a.stride - a.pad;
            next.iw0[pb] = j * a.stride - a.pad;
            next.poff[pb] = next.ih0[pb] * a.W + next.iw0[pb];
        } else {
            next.ih0[pb] = next.iw0[pb] = 0;
            next.poff[pb] = p;
        }
    }
    const int kg0 = wave * a.kg_q + min(wave, a.kg_r);
    next.kg = kg0;
    next.kg_end = kg0 + a.kg_q + (wave < a.kg_r ? 1 : 0);
    {
        const int tap = tdc_div(kg0, a.div_NBk);
        next.dg = kg0 - tap * a.NBk;
        next.r = tdc_div(tap, a.div_K);
        next.s = tap - next.r * a.K;
    }

    tdc_f4 acc[MB][PB];
    TdcPipe<MB, PB, U> pipe;
    TDC_PROBE((MODE - 1) * 5 + 0);
    pipe.start(next);
    TDC_PROBE((MODE - 1) * 5 + 1);
    pipe.run(acc, next.kg_end - kg0, next);
    TDC_PROBE((MODE - 1) * 5 + 2);

    float *__restrict__ outb = a.out + (size_t)b * a.out_rows * a.out_pix;
    tdc_f4 *__restrict__ outb4 = reinterpret_cast<tdc_f4 *>(outb);   // blocked: cell (cb, p, g) = [(cb*out_pix + p)*4 + g]
    if (nw == 1) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) {
                const int p = 16 * (pg * PB + pb) + l16;
                if (a.out_layout == TDC_ACT_BLOCKED) {
                    if (p < a.out_pix) outb4[((size_t)(mg * MB + mb) * a.out_pix + p) * 4 + g] = acc[mb][pb];
                } else if (a.out_layout == TDC_ACT_NHWC) {
                    const int m = 16 * (mg * MB + mb) + 4 * g;
                    if (m < a.out_rows && p < a.out_pix)
                        tdc_store_nhwc(a.out, a.epi, acc[mb][pb], m, ((size_t)b * a.out_pix + p) * a.out_rows + m);
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int m = 16 * (mg * MB + mb) + 4 * g + i;
                        if (m < a.out_rows && p < a.out_pix) {
                            const size_t idx = (size_t)m * a.out_pix + p;
                            outb[idx] = tdc_apply_epilogue(a.epi, acc[mb][pb][i], m, (size_t)b * a.out_rows * a.out_pix + idx);
                        }
                    }
                }
            }
        return;
    }
    // Partial sums of every wavefront to LDS, then a fixed-order sum, one output element per thread.
    constexpr int E = MB * PB * 256;
    if (a.out_layout != TDC_ACT_NCHW) {
        // channel-minor outputs: the partial sums stay as the lanes hold them, [wave][(mb*PB + pb)*64 + lane]
        // 16-byte cells, so that consecutive threads sum and store consecutive channels of one pixel
        tdc_f4 *__restrict__ red4 = reinterpret_cast<tdc_f4 *>(red);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) red4[wave * (E / 4) + (mb * PB + pb) * 64 + lane] = acc[mb][pb];
        __syncthreads();
        TDC_PROBE((MODE - 1) * 5 + 3);
        for (int e = threadIdx.x; e < E; e += blockDim.x) {
            float sum = red[e];
            for (int ww = 1; ww < nw; ++ww) sum += red[ww * E + e];
            const int i = e & 3, ln = (e >> 2) & 63, blk = e >> 8;
            const int pb = blk % PB, mb = blk / PB;
            const int p = 16 * (pg * PB + pb) + (ln & 15);
            if (p >= a.out_pix) continue;
            if (a.out_layout == TDC_ACT_BLOCKED) {
                outb[(((size_t)(mg * MB + mb) * a.out_pix + p) * 4 + (ln >> 4)) * 4 + i] = sum;
            } else {
                const int m = 16 * (mg * MB + mb) + 4 * (ln >> 4) + i;
                if (m < a.out_rows) {
                    const size_t idx = ((size_t)b * a.out_pix + p) * a.out_rows + m;
                    a.out[idx] = tdc_apply_epilogue(a.epi, sum, m, idx);
                }
            }
        }
        TDC_PROBE((MODE - 1) * 5 + 4);
        return;
    }
    // NCHW: [wave][(mb*PB + pb)*4 + i][lane], consecutive threads take consecutive pixels of one channel
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int pb = 0; pb < PB; ++pb)
#pragma unroll
            for (int i = 0; i < 4; ++i) red[wave * E + ((mb * PB + pb) * 4 + i) * 64 + lane] = acc[mb][pb][i];
    __syncthreads();
    TDC_PROBE((MODE - 1) * 5 + 3);
    for (int e = threadIdx.x; e < E; e += blockDim.x) {
        float sum = red[e];
        for (int ww = 1; ww < nw; ++ww) sum += red[ww * E + e];
        const int ln = e & 63, i = (e >> 6) & 3, blk = e >> 8;
        const int pb = blk % PB, mb = blk / PB;
        const int m = 16 * (mg * MB + mb) + 4 * (ln >> 4) + i;
        const int p = 16 * (pg * PB + pb) + (ln & 15);
        if (m < a.out_rows && p < a.out_pix) {
            const size_t idx = (size_t)m * a.out_pix + p;
            outb[idx] = tdc_apply_epilogue(a.epi, sum, m, (size_t)b * a.out_rows * a.out_pix + idx);
        }
    }
    TDC_PROBE((MODE - 1) * 5 + 4);
}

// k-groups fetched per register buffer: 2*U covers up to eight k-groups per wavefront, beyond
// that the choice among the compiled sizes minimises dead MFMA slots in the last buffer.
int pick_u(int kg_per_wave, int umax)
{
    if (kg_per_wave <= 2 * umax) return std::min(umax, std::max(1, (kg_per_wave + 1) / 2));
    int best = umax, waste = 1 << 30;
    for (int u = umax; u >= std::max(1, umax - 1); --u) {
        const int w = (kg_per_wave + u - 1) / u * u - kg_per_wave;
        if (w < waste) {
            waste = w;
            best = u;
        }
    }
    return best;
}

template <int MODE, int ACT>
hipError_t launch_stage(const GemmArgs &a_in, int mb, int pb, int waves, int batch, hipStream_t s)
{
    GemmArgs a = a_in;
    const int n_mgroups = a.NBm / mb;
    a.n_mgroups = n_mgroups;
    // keep the larger operand's re-use inside one XCD: weights when they outweigh the activations
    a.pg_major = (double)a.NBm * a.KG * 1024.0 < (double)a.act_rows_valid * a.act_pix * 4.0;
    a.kg_q = a.KG / waves;
    a.kg_r = a.KG % waves;
    a.div_inner = tdc_make_div((unsigned)(a.pg_major ? n_mgroups : a.n_pgroups));
    a.div_Wo = tdc_make_div((unsigned)a.Wo);
    a.div_NBk = tdc_make_div((unsigned)a.NBk);
    a.div_K = tdc_make_div((unsigned)a.K);
    dim3 grid((unsigned)(n_mgroups * a.n_pgroups), (unsigned)batch), block(64 * waves);
    const size_t lds = waves > 1 ? (size_t)waves * mb * pb * 256 * sizeof(float) : 0;
    const int kg_per_wave = (a.KG + waves - 1) / waves;
    const int umax = mb * pb <= 4 ? 4 : 2;
    int u = pick_u(kg_per_wave, umax);
    if (mb * pb == 4 && u != 4) u = 2;          // compiled sizes: {2,4} for four blocks, {2} beyond
    if (mb * pb > 4) u = 2;
#define TDC_CASE(M_, P_, U_)                                                                      \
    if (mb == M_ && pb == P_ && u == U_) {                                                        \
        hipLaunchKernelGGL((tdc_gemm_kernel<MODE, ACT, M_, P_, U_>), grid, block, lds, s, a);    \
        return hipGetLastError();                                                                 \
    }
    TDC_CASE(1, 1, 1) TDC_CASE(1, 1, 2) TDC_CASE(1, 1, 3) TDC_CASE(1, 1, 4)
    TDC_CASE(2, 1, 1) TDC_CASE(2, 1, 2) TDC_CASE(2, 1, 3) TDC_CASE(2, 1, 4)
    TDC_CASE(1, 2, 1) TDC_CASE(1, 2, 2) TDC_CASE(1, 2, 3) TDC_CASE(1, 2, 4)
    TDC_CASE(2, 2, 2) TDC_CASE(2, 2, 4) TDC_CASE(4, 1, 2) TDC_CASE(4, 1, 4) TDC_CASE(1, 4, 2) TDC_CASE(1, 4, 4)
    TDC_CASE(4, 2, 2) TDC_CASE(2, 4, 2) TDC_CASE(4, 4, 2)
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
                            float *z1, float *z2, float *y, const TdcEpi &epi)
{
    const int HW = d.H * d.W, P = d.Ho * d.Wo;
    GemmArgs a;
    a.epi = TdcEpi{nullptr, nullptr, 0};
    // stage 1 (Eq. 2): z1 = U_in^T x
    a.act = x; a.wp = uin_p; a.out = z1;
    a.act_rows = d.C; a.act_rows_valid = d.C; a.act_pix = HW;
    a.out_rows = 16 * d.NB1; a.out_pix = HW; a.out_layout = TDC_ACT_BLOCKED;
    a.NBm = d.NB1; a.KG = d.KG1; a.NBk = 1;
    a.n_pgroups = ((HW + 15) / 16 + t.pb[0] - 1) / t.pb[0];
    a.H = d.H; a.W = d.W; a.Wo = d.Wo; a.K = d.K; a.stride = d.stride; a.pad = d.pad;
    hipError_t e = d.nhwc ? launch_stage<1, TDC_ACT_NHWC>(a, t.mb[0], t.pb[0], t.waves[0], d.B, s)
                          : launch_stage<1, TDC_ACT_NCHW>(a, t.mb[0], t.pb[0], t.waves[0], d.B, s);
    if (e != hipSuccess) return e;
    // stage 2 (Eq. 3): z2 = core conv of z1
    a.act = z1; a.wp = core_p; a.out = z2;
    a.act_rows = 16 * d.NB1; a.act_rows_valid = 16 * d.NB1; a.act_pix = HW;
    a.out_rows = 16 * d.NB2; a.out_pix = P; a.out_layout = TDC_ACT_BLOCKED;
    a.NBm = d.NB2; a.KG = d.K * d.K * d.NB1; a.NBk = d.NB1;
    a.n_pgroups = ((P + 15) / 16 + t.pb[1] - 1) / t.pb[1];
    e = launch_stage<2, TDC_ACT_BLOCKED>(a, t.mb[1], t.pb[1], t.waves[1], d.B, s);
    if (e != hipSuccess) return e;
    // stage 3 (Eq. 4): y = U_out^T z2
    a.act = z2; a.wp = uout_p; a.out = y;
    a.act_rows = 16 * d.NB2; a.act_rows_valid = 16 * d.NB2; a.act_pix = P;
    a.out_rows = d.N; a.out_pix = P; a.out_layout = d.nhwc ? TDC_ACT_NHWC : TDC_ACT_NCHW; a.epi = epi;
    a.NBm = d.NB3; a.KG = d.NB2; a.NBk = 1;
    a.n_pgroups = ((P + 15) / 16 + t.pb[2] - 1) / t.pb[2];
    return launch_stage<3, TDC_ACT_BLOCKED>(a, t.mb[2], t.pb[2], t.waves[2], d.B, s);
}

// The undecomposed layer (Eq. 1's kernel applied directly): the stage-2 implicit GEMM with the
// layer's own channels in place of the ranks.  `d` carries R1 = C and R2 = N, so NB1 counts the
// 16-blocks of C and NB2 those of N; x has exactly C rows (rows of the last, partial block lie
// beyond the buffer descriptor and read as zero) and y exactly N.
hipError_t tdc_launch_dense(const TdcDims &d, const tdc_tuning &t, hipStream_t s, const float *x,
                            const float *w_p, float *y, const TdcEpi &epi)
{
    const int HW = d.H * d.W, P = d.Ho * d.Wo;
    GemmArgs a;
    a.epi = TdcEpi{nullptr, nullptr, 0};
    a.act = x; a.wp = w_p; a.out = y;
    a.act_rows = d.C; a.act_rows_valid = d.C; a.act_pix = HW;
    a.out_rows = d.N; a.out_pix = P; a.out_layout = d.nhwc ? TDC_ACT_NHWC : TDC_ACT_NCHW; a.epi = epi;
    a.NBm = d.NB2; a.KG = d.K * d.K * d.NB1; a.NBk = d.NB1;
    a.n_pgroups = ((P + 15) / 16 + t.pb[1] - 1) / t.pb[1];
    a.H = d.H; a.W = d.W; a.Wo = d.Wo; a.K = d.K; a.stride = d.stride; a.pad = d.pad;
    return d.nhwc ? launch_stage<2, TDC_ACT_NHWC>(a, t.mb[1], t.pb[1], t.waves[1], d.B, s)
                  : launch_stage<2, TDC_ACT_NCHW>(a, t.mb[1], t.pb[1], t.waves[1], d.B, s);
}

// MERGED variant: two launches.  Stage 1 as in SPLIT; then one implicit GEMM R1 -> N with the
// kernel Wm = core x_2 U_out (stage 3 folded into the core when the weights are re-laid out).  It
// spends K*K*R1*N instead of K*K*R1*R2 + R2*N MACs per output pixel, but its output-channel
// blocks are independent workgroups, which is what a small image lacks, and a launch is saved.
hipError_t tdc_launch_merged(const TdcDims &d, const tdc_tuning &t, hipStream_t s, const float *x,
                             const float *uin_p, const float *wm_p, float *z1, float *y, const TdcEpi &epi)
{
    const int HW = d.H * d.W, P = d.Ho * d.Wo;
    GemmArgs a;
    a.epi = TdcEpi{nullptr, nullptr, 0};
    a.act = x; a.wp = uin_p; a.out = z1;
    a.act_rows = d.C; a.act_rows_valid = d.C; a.act_pix = HW;
    a.out_rows = 16 * d.NB1; a.out_pix = HW; a.out_layout = TDC_ACT_BLOCKED;
    a.NBm = d.NB1; a.KG = d.KG1; a.NBk = 1;
    a.n_pgroups = ((HW + 15) / 16 + t.pb[0] - 1) / t.pb[0];
    a.H = d.H; a.W = d.W; a.Wo = d.Wo; a.K = d.K; a.stride = d.stride; a.pad = d.pad;
    hipError_t e = d.nhwc ? launch_stage<1, TDC_ACT_NHWC>(a, t.mb[0], t.pb[0], t.waves[0], d.B, s)
                          : launch_stage<1, TDC_ACT_NCHW>(a, t.mb[0], t.pb[0], t.waves[0], d.B, s);
    if (e != hipSuccess) return e;
    a.act = z1; a.wp = wm_p; a.out = y;
    a.act_rows = 16 * d.NB1; a.act_rows_valid = 16 * d.NB1; a.act_pix = HW;
    a.out_rows = d.N; a.out_pix = P; a.out_layout = d.nhwc ? TDC_ACT_NHWC : TDC_ACT_NCHW; a.epi = epi;
    a.NBm = d.NB3; a.KG = d.K * d.K * d.NB1; a.NBk = d.NB1;
    a.n_pgroups = ((P + 15) / 16 + t.pb[1] - 1) / t.pb[1];
    return launch_stage<2, TDC_ACT_BLOCKED>(a, t.mb[1], t.pb[1], t.waves[1], d.B, s);
}
