// CHAIN variant: the fused kernel for the throughput regime.  Like FUSED, one workgroup evaluates
// all three stages (Eqs. 2, 3, 4) for one TH x TW output tile of one image with the z1 tile and
// its halo in LDS.  Unlike FUSED, stages 2 and 3 are chained inside a wavefront:
//
//   - a wavefront owns whole groups of 16-pixel blocks of the output tile and computes ALL R2
//     channels of z2 for them (NB2 = R2P/16 is a template parameter so that the NB2 x PB
//     accumulator blocks live in registers; every z1 operand read from LDS is used NB2 times);
//   - with the k-order of tdc_mfma.h those accumulator registers are, as they stand, the operand
//     of stage 3, so z2 never goes through LDS and there is no barrier between stages 2 and 3;
//   - stage 3 runs with the MFMA operands swapped, D = z2^T U_out, which leaves each lane with
//     four consecutive PIXELS of one output channel: y is written with one 16-byte buffer store
//     per lane instead of four 4-byte stores of four channels (scalar stores when the tile or
//     image width is not a multiple of 4).  With NHWC activations (template flag) the operands
//     stay unswapped instead: a lane then holds four consecutive CHANNELS of one pixel, which is
//     the 16-byte store of that layout, and stage 1 reads x with one 16-byte load per lane.
//
// The paper's kernel keeps one output channel per thread and the R x S weights of the current
// input channel in registers (section 5.2); here the register-resident object is the whole
// R2-channel column of z2 for 16 or 32 pixels, which is what lets the 1x1 expansion ride along.
#ifndef TDC_CHAIN_KERNEL_H
#define TDC_CHAIN_KERNEL_H

#include <type_traits>

#include "tdc_internal.h"
#include "tdc_mfma.h"
#include "tdc_stage1.h"

struct TdcChainArgs {
    const float *x, *uin_p, *core_p, *uout_p;
    float *y;
    int C, N, H, W, Ho, Wo, K, stride, pad;
    int NB1, NB3, KG1;
    int TH, TW, QW, Q, P, QB, PBk;
    int tiles_x;
    int pitch1;             // LDS row pitch of the z1 tile, in 16-byte cells
    int w_core4, w_uout4;   // 16-byte units of the packed core / U_out arrays
    int QH, RPR, n_sb;      // run-major stage 1: tile rows, runs per row, 64-pixel blocks of runs
    TdcDiv div_RPR;
    int vec;                // 1: tile width, image width and tile origin are multiples of 4 -> 16-byte stores
    TdcEpi epi;
    TdcDiv div_tiles_x, div_QW, div_TW, div_tiles;   // launch-time constant divisors
    int tiles, xcd_per, xcd_rem;   // tiles per image; workgroups per XCD (and the remainder) of the id remap
    unsigned inv_mg1;       // ceil(2^20 / (NB1 / mb1)): divides a stage-1 unit index by the channel groups
};

namespace {


__device__ __forceinline__ void tdc_buf_store(tdc_rsrc r, unsigned byte_off, float v)
{
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), r, (int)byte_off, 0, 0);
}

__device__ __forceinline__ void tdc_buf_store4(tdc_rsrc r, unsigned byte_off, tdc_f4 v)
{
    typedef unsigned u4 __attribute__((ext_vector_type(4)));
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4, v), r, (int)byte_off, 0, 0);
}

// Stage 1 (Eq. 2) for the whole workgroup: z1 tile = U_in^T x into LDS cells, and the weights of
// stages 2 and 3 into LDS when they fit (their first loads travel while stage 1 computes).
template <int MB1, int PB, int LAY>
__device__ __forceinline__ void chain_stage1(const TdcChainArgs &a, tdc_f4 *__restrict__ z1s, int lane, int wave, int nw,
                                             int b, int h0, int w0, tdc_f4 *__restrict__ wC, bool copy_weights)
{
    TdcS1Geom sg;
    sg.x_img = a.x + (size_t)b * a.C * a.H * a.W; sg.uin_p = a.uin_p;
    sg.C = a.C; sg.H = a.H; sg.W = a.W; sg.KG1 = a.KG1; sg.NB1 = a.NB1;
    sg.QB = a.QB; sg.Q = a.Q; sg.QW = a.QW; sg.h0 = h0; sg.w0 = w0; sg.pitch1 = a.pitch1;
    sg.div_QW = a.div_QW; sg.inv_mg = a.inv_mg1;
    sg.QH = a.QH; sg.RPR = a.RPR; sg.n_sb = a.n_sb; sg.div_RPR = a.div_RPR;
    const tdc_f4 *__restrict__ core4 = reinterpret_cast<const tdc_f4 *>(a.core_p);
    const tdc_f4 *__restrict__ uout4 = reinterpret_cast<const tdc_f4 *>(a.uout_p);
    const auto stage1 = [&](auto &s1) {
        s1.prefetch();
        TdcWeightCopy<8> wc;
        if (copy_weights) wc.load(core4, a.w_core4, uout4, a.w_uout4, 0);
        s1.zero_outside(z1s);
        s1.run(z1s);
        if (copy_weights) {
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
        TdcStage1<MB1, PB, (MB1 * PB >= 8 ? 2 : 4), LAY == TDC_LAY_NHWC> s1(sg, lane, wave, nw);   // k-groups per operand buffer
        stage1(s1);
    }
}

// (Asking the compiler for four wavefronts per SIMD on the run-major instances that need 137 registers makes them
// spill 36 bytes per lane and run 5 % slower alone; they stay at three.)
template <int NB2, int PB, bool WLDS, int LAY, int MB1>
__global__ __launch_bounds__(512) void tdc_chain_kernel(TdcChainArgs a)
{
    constexpr bool NHWC = LAY == TDC_LAY_NHWC;
    extern __shared__ tdc_f4 lds4[];
    tdc_f4 *__restrict__ z1s = lds4;                                  // [NB1][4][pitch1]
    tdc_f4 *__restrict__ wC = z1s + (size_t)4 * a.NB1 * a.pitch1;     // packed core   (WLDS)
    tdc_f4 *__restrict__ wO = wC + a.w_core4;                         // packed U_out  (WLDS)

    // every argument stage 1 needs, in one round of scalar loads (see TDC_FETCH_NOW)
    unsigned bd = blockDim.x;
    TdcDiv div_tiles_x = a.div_tiles_x;
    TDC_FETCH_NOW(TDC_OUTS("+s"(bd), "+s"(div_tiles_x.m)), "s"(a.x), "s"(a.uin_p), "s"(a.core_p), "s"(a.uout_p), "s"(a.y), "s"(a.C), "s"(a.H), "s"(a.W),
                  "s"(a.stride), "s"(a.pad), "s"(a.NB1), "s"(a.KG1), "s"(a.TH), "s"(a.TW), "s"(a.QW), "s"(a.Q), "s"(a.QB), "s"(a.tiles_x),
                  "s"(a.pitch1), "s"(a.w_core4), "s"(a.w_uout4), "s"(a.QH), "s"(a.RPR), "s"(a.n_sb), "s"(a.div_RPR.m), "s"(a.div_RPR.sh1),
                  "s"(a.div_RPR.sh2), "s"(div_tiles_x.sh1), "s"(div_tiles_x.sh2),
                  "s"(a.div_QW.m), "s"(a.div_QW.sh1), "s"(a.div_QW.sh2), "s"(a.inv_mg1), "s"(a.tiles), "s"(a.xcd_per),
                  "s"(a.xcd_rem), "s"(a.div_tiles.m), "s"(a.div_tiles.sh1), "s"(a.div_tiles.sh2));
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

    TDC_PROBE(0);
    // ------------------------------------------------------------------ stage 1 (Eq. 2)
    {
        chain_stage1<MB1, PB, LAY>(a, z1s, lane, wave, nw, b, h0, w0, wC, WLDS);
    }
    TDC_PROBE(3);
    __syncthreads();
    TDC_PROBE(4);

    // ------------------------------------------------- stages 2 and 3 (Eqs. 3, 4), per wavefront
    const int KG2 = a.K * a.K * a.NB1;
    const int P2 = a.Ho * a.Wo;
    const tdc_rsrc crs = tdc_make_rsrc(a.core_p, (unsigned)a.w_core4 * 16u);
    const tdc_rsrc ors = tdc_make_rsrc(a.uout_p, (unsigned)a.w_uout4 * 16u);
    const tdc_rsrc yrs = tdc_make_rsrc(a.y + (size_t)b * a.N * P2, (unsigned)a.N * P2 * 4u);
    const int n_pg = (a.PBk + PB - 1) / PB;
    for (int pg = wave; pg < n_pg; pg += nw) {
        // ---- stage 2: acc2[kg2][pb] = z2 channels 16*kg2 + 4*g + {0..3} of pixel l16 of block pb
        int qbase[PB];
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
            const int p = 16 * (pg * PB + pb) + l16;
            const int ph = tdc_div(p, a.div_TW), pw = p - ph * a.TW;
            qbase[pb] = g * a.pitch1 + (p < a.P ? ph * a.stride * a.QW + pw * a.stride : 0);
        }
        tdc_f4 acc2[NB2][PB];
        {
            // weights streamed from L2 (they did not fit in LDS) need two k-groups of lookahead to cover
            // its latency; a dead k-group then multiplies zeros (the buffer load returns 0)
            constexpr int U = (WLDS || NB2 > 4) ? 1 : 2;
            int kg = 0, dg = 0, s = 0, toff = 0;     // toff = r*QW + s
            auto next = [&](tdc_f4(&av)[NB2], tdc_f4(&bv)[PB]) {
                const bool live = kg < KG2;
#pragma unroll
                for (int mb = 0; mb < NB2; ++mb) {
                    const int frag = mb * KG2 + kg;
                    // WLDS: a dead fetch is never multiplied (one k-group per buffer); it only has to stay in range
                    if (WLDS) av[mb] = wC[(live ? frag : 0) * 64 + lane];
                    else av[mb] = tdc_buf_load4(crs, ((unsigned)frag * 1024u + lane * 16u) | (live ? 0u : TDC_OOB));
                }
                const int cell = live ? dg * 4 * a.pitch1 + toff : 0;
#pragma unroll
                for (int pb = 0; pb < PB; ++pb) bv[pb] = z1s[cell + qbase[pb]];
                ++kg;
                // position of the next k-group inside (tap, 16-channel group of z1), without branches
                const int nd = dg + 1;
                const bool w1 = nd == a.NB1;
                dg = w1 ? 0 : nd;
                const int ns = s + (w1 ? 1 : 0);
                const bool w2 = ns == a.K;
                s = w2 ? 0 : ns;
                toff += (w1 ? 1 : 0) + (w2 ? a.QW - a.K : 0);
            };
            TdcPipe<NB2, PB, U> pipe;
            pipe.start(next);
            pipe.run(acc2, KG2, next);
        }
        TDC_PROBE(5);
        // ---- stage 3.  NCHW: D[pixel 4*g + i][channel l16] = sum_d2 z2[d2][pixel] * U_out[d2][channel];
        //      NHWC: D[channel 4*g + i][pixel l16], the same products with the operands unswapped
        unsigned yq[PB][4];      // NCHW: byte offset of pixel 4*g + i of block pb in one channel plane, or TDC_OOB
        int ypix[PB];            // NHWC: index of pixel l16 of block pb in the output image, or -1
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int p = 16 * (pg * PB + pb) + 4 * g + i;
                const int ph = tdc_div(p, a.div_TW), pw = p - ph * a.TW;
                const int oi = i0 + ph, oj = j0 + pw;
                yq[pb][i] = (p < a.P && oi < a.Ho && oj < a.Wo) ? (unsigned)(oi * a.Wo + oj) * 4u : TDC_OOB;
            }
            const int p = 16 * (pg * PB + pb) + l16;
            const int ph = tdc_div(p, a.div_TW), pw = p - ph * a.TW;
            const int oi = i0 + ph, oj = j0 + pw;
            ypix[pb] = (p < a.P && oi < a.Ho && oj < a.Wo) ? oi * a.Wo + oj : -1;
        }
        constexpr int D3 = (WLDS || NB2 > 4) ? 2 : 3;     // U_out blocks in flight (from L2: one more)
        tdc_f4 ua[D3][NB2];
        const auto fetch = [&](int nb, tdc_f4(&u)[NB2]) {
            const bool live = nb < a.NB3;
#pragma unroll
            for (int kg = 0; kg < NB2; ++kg) {
                const int frag = nb * NB2 + kg;
                if (WLDS) u[kg] = wO[(live ? frag : 0) * 64 + lane];
                else u[kg] = tdc_buf_load4(ors, ((unsigned)frag * 1024u + lane * 16u) | (live ? 0u : TDC_OOB));
            }
        };
        // `with_epi` is a compile-time flag: the loop over output blocks exists twice, with and without the epilogue.
        // The epilogue loads (bias, shortcut) put vector-memory loads into the loop, and the waits the compiler
        // then needs before reusing their registers count the y stores of the previous block as well (stores and
        // loads share one in-order counter): every block would wait for the stores of the one before it.  The
        // plain loop has stores only and never waits on them.
        const auto emit = [&](auto with_epi, int nb, const tdc_f4(&u)[NB2]) {
            constexpr bool EPI = decltype(with_epi)::value;
            tdc_f4 acc3[PB];
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) acc3[pb] = tdc_f4_zero();
#pragma unroll
            for (int kg = 0; kg < NB2; ++kg)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int pb = 0; pb < PB; ++pb)
                        acc3[pb] = NHWC ? tdc_mfma(u[kg][j], acc2[kg][pb][j], acc3[pb]) : tdc_mfma(acc2[kg][pb][j], u[kg][j], acc3[pb]);
            if (NHWC) {
                const int n = 16 * nb + 4 * g;
#pragma unroll
                for (int pb = 0; pb < PB; ++pb)
                    if (ypix[pb] >= 0 && n < a.N) {
                        const size_t cell = ((size_t)b * P2 + ypix[pb]) * a.N + n;
                        if constexpr (EPI) tdc_store_nhwc<true>(a.y, a.epi, acc3[pb], n, cell);
                        else tdc_store4_stream(reinterpret_cast<tdc_f4 *>(a.y + cell), acc3[pb]);
                    }
                return;
            }
            // channels past N lie beyond the descriptor: the hardware drops those stores
            const unsigned plane = (unsigned)(16 * nb + l16) * P2 * 4u;
            if constexpr (EPI) {
                // this lane holds channel 16*nb + l16 at the four pixels 4*g + i of every block
                const int n = 16 * nb + l16;
                const float bias = (a.epi.bias && n < a.N) ? a.epi.bias[n] : 0.f;
#pragma unroll
                for (int pb = 0; pb < PB; ++pb)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        float v = acc3[pb][i] + bias;
                        if (a.epi.residual && n < a.N && !(yq[pb][i] & TDC_OOB))
                            v += a.epi.residual[(size_t)b * a.N * P2 + (size_t)n * P2 + (yq[pb][i] >> 2)];
                        acc3[pb][i] = a.epi.relu ? fmaxf(v, 0.f) : v;
                    }
            }
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) {
                if (a.vec) {
                    tdc_buf_store4(yrs, (plane + yq[pb][0]) | (yq[pb][0] & TDC_OOB), acc3[pb]);
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        tdc_buf_store(yrs, (plane + yq[pb][i]) | (yq[pb][i] & TDC_OOB), acc3[pb][i]);
                }
            }
        };
        const auto stage3 = [&](auto with_epi) {
            fetch(0, ua[0]);
            if constexpr (D3 == 3) {
                fetch(1, ua[1]);
                for (int nb = 0; nb < a.NB3; nb += 3) {
                    fetch(nb + 2, ua[2]);
                    emit(with_epi, nb, ua[0]);
                    fetch(nb + 3, ua[0]);
                    if (nb + 1 < a.NB3) emit(with_epi, nb + 1, ua[1]);
                    fetch(nb + 4, ua[1]);
                    if (nb + 2 < a.NB3) emit(with_epi, nb + 2, ua[2]);
                }
            } else {
                for (int nb = 0; nb < a.NB3; nb += 2) {
                    fetch(nb + 1, ua[1]);
                    emit(with_epi, nb, ua[0]);
                    fetch(nb + 2, ua[0]);
                    if (nb + 1 < a.NB3) emit(with_epi, nb + 1, ua[1]);
                }
            }
        };
        if (a.epi.bias || a.epi.residual || a.epi.relu) stage3(std::true_type{});
        else stage3(std::false_type{});
    }
    TDC_PROBE(7);
}

#define TDC_CHAIN_NB2(X) X(1) X(2) X(3) X(4) X(5) X(6) X(8) X(10)

}  // namespace

// Launch (or, with prepare_only, only prepare) the instance for stage-1 register tiles of MB1 channel blocks.  MB1 is a
// template parameter of the kernel, not a run-time switch inside it: an instance then carries the registers of one
// stage-1 form only (a kernel holding all three needed 137-246 against 82-196), which is what decides how many
// workgroups a compute unit can hold.  Each MB1 lives in a translation unit of its own (tdc_chain_mb*.hip).
template <int MB1>
hipError_t tdc_launch_chain_instance(const TdcChainArgs &a, int nb2, int pb, bool weights_in_lds, int lay, dim3 grid, dim3 block,
                                     size_t lds_bytes, hipStream_t s, bool prepare_only)
{
#define TDC_LAUNCH(N_, P_, W_, L_)                                                                     \
    {                                                                                                  \
        {                                                                                              \
            hipError_t e = tdc_allow_lds((const void *)tdc_chain_kernel<N_, P_, W_, L_, MB1>, lds_bytes);    \
            if (e != hipSuccess) return e;                                                             \
            if (prepare_only) return hipSuccess;                                                       \
        }                                                                                              \
        hipLaunchKernelGGL((tdc_chain_kernel<N_, P_, W_, L_, MB1>), grid, block, lds_bytes, s, a);     \
        return hipGetLastError();                                                                      \
    }
#define TDC_LAYOUT(N_, P_, W_)                                                                         \
    {                                                                                                  \
        if (lay == TDC_LAY_NHWC) TDC_LAUNCH(N_, P_, W_, TDC_LAY_NHWC)                                  \
        else if (lay == TDC_LAY_NCHW_RUNS) TDC_LAUNCH(N_, P_, W_, TDC_LAY_NCHW_RUNS)                   \
        else TDC_LAUNCH(N_, P_, W_, TDC_LAY_NCHW)                                                      \
    }
#define TDC_X(N_)                                                                                      \
    if (nb2 == N_) {                                                                                   \
        if (pb == 1) {                                                                                 \
            if (weights_in_lds) TDC_LAYOUT(N_, 1, true) else TDC_LAYOUT(N_, 1, false)                  \
        } else {                                                                                       \
            if (weights_in_lds) TDC_LAYOUT(N_, 2, true) else TDC_LAYOUT(N_, 2, false)                  \
        }                                                                                              \
    }
    TDC_CHAIN_NB2(TDC_X)
#undef TDC_X
#undef TDC_LAYOUT
#undef TDC_LAUNCH
    return hipErrorInvalidValue;
}

#endif
