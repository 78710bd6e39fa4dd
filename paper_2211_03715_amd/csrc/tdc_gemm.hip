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

// ---- MERGED in one launch.  What the two-launch form loses at batch 1 is the boundary between its kernels (the
// write-back at the end of the first, the dispatch of the second, its first loads: 1.7-2.3 us of a 7-9 us layer).
// Here the workgroups that run on one XCD -- they share its L2 -- first compute stage 1 (Eq. 2) together, all of
// it, into a copy of z1 that belongs to their XCD (stage 1 is done once per XCD, eight times in all: it is a ninth
// of the layer's work at these shapes and there is no cheaper way to put z1 into every L2), meet at a barrier
// among themselves, and then run their share of the merged K x K GEMM on that copy.  Nothing crosses an XCD inside
// the launch, so no L2 write-back is needed: a wavefront waits for its own stores (they are then in the L2, the
// L1 being write-through), the workgroup bumps its arrival word, and one wavefront polls the arrival words of its
// XCD with loads that miss the L1.  z1 is read by nobody before the barrier, so plain loads see it afterwards.
//   The XCD of a workgroup is read from the hardware (XCC_ID), never inferred; its role among the workgroups of
// that XCD is blockIdx.x / 8, which assumes what the XCD-aware numbering elsewhere in this library assumes for
// speed only: workgroups are dealt to the 8 XCDs round-robin.  Were that ever not so, a role would be missing on
// some XCD and its arrival word would lag.  The wait is bounded for that case and for the likelier one that some
// workgroups of the launch are not resident yet (other streams' kernels hold their compute units): a workgroup
// that has waited long enough computes all of stage 1 for its XCD itself and goes on -- slower, the same bits, and
// no workgroup ever depends on another for more than time.  Arrival words count calls (each workgroup adds one to
// its own word), so nothing depends on host state and a captured graph can be replayed.
//   Units are single 16x16 output blocks; tw1 (tw2) wavefronts of a workgroup split the contraction of a unit and
// add their partial sums through LDS in a fixed order, as in the kernel above; 8/tw teams work side by side.
struct XcdArgs {
    const float *x, *uin_p, *wm_p;
    float *z1c;            // 8 copies of z1, blocked layout, z1_stride floats apart
    float *y;
    unsigned *arrive;      // [8 XCDs][32 roles], then one word that counts the waits given up
    unsigned *status;      // host-visible; set non-zero by a kernel that finds XCD or role numbers it does not know
    TdcEpi epi;
    unsigned z1_stride, wait_limit;
    int C, N, HW, P, NB1, NB3, KG1, KG2, H, W, Wo, K, stride, pad;
    int lg1, lg2;          // log2 of the wavefronts per team in stage 1 / in the merged GEMM
    int q1, rem1, q2, rem2;   // k-groups per wavefront of a team: the first rem take q + 1
    int n1, n2, npb1, npb2, Wn, rounds1, rounds2, nhwc;
    TdcDiv div_Wo, div_NBk, div_K, div_npb1, div_npb2, div_NB1, div_NB3;
};

// NK > 0: the merged GEMM takes one pass (every team has at most one unit) and a wavefront at most NK k-groups of
// it.  Its weight fragments are then requested at the very start of the kernel and wait in registers, so that
// behind the barrier only the z1 loads and the MFMAs remain.
// NK == 0: any size, operands streamed through TdcPipe as in the GEMM kernel.
template <int ACT, int NK>
__global__ __launch_bounds__(512) void tdc_merged_xcd_kernel(XcdArgs a)
{
    __shared__ float red[8 * 256];
    __shared__ int go;
    constexpr int U = 4;
    // the kernel arguments span several cache lines of host-visible memory: ask for all of them now, at once
    TDC_FETCH_NOW(TDC_OUTS("+s"(a.z1_stride), "+s"(a.wait_limit)), "s"(a.x), "s"(a.uin_p), "s"(a.wm_p), "s"(a.z1c), "s"(a.y),
                  "s"(a.arrive), "s"(a.epi.bias), "s"(a.epi.residual), "s"(a.epi.relu), "s"(a.C), "s"(a.N), "s"(a.HW), "s"(a.P),
                  "s"(a.NB1), "s"(a.NB3), "s"(a.KG1), "s"(a.KG2), "s"(a.H), "s"(a.W), "s"(a.Wo), "s"(a.K), "s"(a.stride),
                  "s"(a.pad), "s"(a.lg1), "s"(a.lg2), "s"(a.q1), "s"(a.rem1), "s"(a.q2), "s"(a.rem2), "s"(a.n1), "s"(a.n2), "s"(a.npb1), "s"(a.npb2), "s"(a.Wn), "s"(a.rounds1),
                  "s"(a.rounds2), "s"(a.nhwc), "s"(a.div_Wo.m), "s"(a.div_Wo.sh1), "s"(a.div_Wo.sh2), "s"(a.div_NBk.m),
                  "s"(a.div_NBk.sh1), "s"(a.div_NBk.sh2), "s"(a.div_K.m), "s"(a.div_K.sh1), "s"(a.div_K.sh2), "s"(a.div_npb1.m),
                  "s"(a.div_npb1.sh1), "s"(a.div_npb1.sh2), "s"(a.div_npb2.m), "s"(a.div_npb2.sh1), "s"(a.div_npb2.sh2),
                  "s"(a.div_NB1.m), "s"(a.div_NB1.sh1), "s"(a.div_NB1.sh2), "s"(a.div_NB3.m), "s"(a.div_NB3.sh1), "s"(a.div_NB3.sh2));
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, l16 = lane & 15;
    unsigned xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    xcc &= 15u;
    const int role = blockIdx.x >> 3;
    TDC_PROBE(0);
    if (xcc >= 8u || role >= 32) {   // not the chip this kernel was written for
        if (threadIdx.x == 0) __hip_atomic_store(a.status, 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        return;
    }
    unsigned *my_arrive = a.arrive + xcc * 32;
    const tdc_rsrc ars_flags = tdc_make_rsrc(my_arrive, 32 * 4);
    unsigned own = 0;   // this workgroup's own arrival word as the call before left it; loaded behind stage 1's first operands
    float *z1x = a.z1c + (size_t)xcc * a.z1_stride;
    tdc_f4 *__restrict__ red4 = reinterpret_cast<tdc_f4 *>(red);

    // ---- what the second phase will need (NK > 0: its single unit), worked out before anything waits
    const int G = (int)gridDim.x;
    const int tw2 = 1 << a.lg2, teams2 = 8 >> a.lg2, team2 = wave >> a.lg2, wt2 = wave & (tw2 - 1);
    const int q2 = a.q2, rem2 = a.rem2;
    const int lw = tdc_logical_block(blockIdx.x, G);
    const int kg02 = wt2 * q2 + min(wt2, rem2);
    int tap0, dg0, r0, s0;
    {
        tap0 = tdc_div(kg02, a.div_NBk);
        dg0 = kg02 - tap0 * a.NB1;
        r0 = tdc_div(tap0, a.div_K);
        s0 = tap0 - r0 * a.K;
    }
    tdc_f4 wk[NK > 0 ? NK : 1];
    int u2 = 0, b2 = 0, mg2 = 0, pg2 = 0, cnt2 = 0, ih2 = 0, iw2 = 0;
    bool live2 = false;
    // ---- stage 1, all of it, by the workgroups of this XCD (pass 0); by this workgroup alone if the others did not
    // show up at the barrier in time (pass 1, see there)
    int role1 = role, wn1 = a.Wn, rounds1 = a.rounds1;
    for (int pass = 0;; ++pass) {
        const int tw = 1 << a.lg1, teams = 8 >> a.lg1, team = wave >> a.lg1, wt = wave & (tw - 1);
        const int q = a.q1, rem = a.rem1;
        for (int r = 0; r < rounds1; ++r) {
            const int u = (r * wn1 + role1) * teams + team;
            const bool live = u < a.n1;
            const int pgb = tdc_div(live ? u : 0, a.div_NB1), mg = (live ? u : 0) - pgb * a.NB1;   // (b, pixel group), channel block
            const int b = tdc_div(pgb, a.div_npb1), pg = pgb - b * a.npb1;
            GemmNext<1, ACT, 1, 1> next;
            next.wstride = 0;
            next.wrs = tdc_make_rsrc(a.uin_p + (size_t)mg * a.KG1 * 256, (unsigned)a.KG1 * 1024u);
            next.ars = tdc_make_rsrc(a.x + (size_t)b * a.C * a.HW, (unsigned)a.C * a.HW * 4u);
            next.wlane = lane * 16u;
            next.act_pix = a.HW; next.C = a.C; next.NBk = 1; next.K = a.K; next.H = a.H; next.W = a.W; next.g = g;
            const int p = 16 * pg + l16;
            next.pval[0] = p < a.HW; next.ih0[0] = next.iw0[0] = 0; next.poff[0] = p;
            const int kg0 = wt * q + min(wt, rem);
            next.kg = kg0;
            next.kg_end = live ? kg0 + q + (wt < rem ? 1 : 0) : kg0;
            next.dg = next.r = next.s = 0;
            tdc_f4 acc[1][1];
            TdcPipe<1, 1, U> pipe;
            pipe.start(next);
            TDC_PROBE(1);
            // written by this workgroup (same XCD, same role) in the call before: one more than it is the value to reach.
            // Every wavefront loads it, and here: a load in front of the loop, or inside a branch only wavefront 0 takes,
            // is waited for on the spot, a memory round trip before the first operand is even requested.
            if (r == 0 && pass == 0) own = (unsigned)__builtin_amdgcn_raw_buffer_load_b32(ars_flags, role * 4, 0, 16);
            if (NK > 0 && r == 0 && pass == 0) {
                u2 = lw * teams2 + team2;
                live2 = u2 < a.n2;
                const int bm = tdc_div(live2 ? u2 : 0, a.div_npb2);
                pg2 = (live2 ? u2 : 0) - bm * a.npb2;
                b2 = tdc_div(bm, a.div_NB3);
                mg2 = bm - b2 * a.NB3;
                cnt2 = live2 ? q2 + (wt2 < rem2 ? 1 : 0) : 0;
                const int p = 16 * pg2 + l16;
                const int i = tdc_div(p, a.div_Wo), j = p - i * a.Wo;
                ih2 = i * a.stride - a.pad;
                iw2 = j * a.stride - a.pad;
                // the merged GEMM's weight fragments of this wavefront, requested right behind the first operands of
                // stage 1: they come from HBM (every workgroup has its own) and have all of stage 1 to arrive
                const tdc_rsrc wrs2 = tdc_make_rsrc(a.wm_p + (size_t)mg2 * a.KG2 * 256, (unsigned)a.KG2 * 1024u);
#pragma unroll
                for (int k = 0; k < NK; ++k)
                    wk[k] = tdc_buf_load4(wrs2, ((unsigned)(kg02 + k) * 1024u + lane * 16u) | (k < cnt2 ? 0u : TDC_OOB));
            }
            pipe.run(acc, next.kg_end - kg0, next);
            TDC_PROBE(2);
            tdc_f4 *__restrict__ z14 = reinterpret_cast<tdc_f4 *>(z1x + (size_t)b * 16 * a.NB1 * a.HW);
            if (tw == 1) {
                if (live && p < a.HW) z14[((size_t)mg * a.HW + p) * 4 + g] = acc[0][0];
            } else {
                red4[wave * 64 + lane] = acc[0][0];
                __syncthreads();
                for (int e = wt * 64 + lane; e < 256; e += tw * 64) {
                    float sum = red[team * tw * 256 + e];
                    for (int ww = 1; ww < tw; ++ww) sum += red[(team * tw + ww) * 256 + e];
                    const int i = e & 3, ln = (e >> 2) & 63;
                    const int pp = 16 * pg + (ln & 15);
                    if (live && pp < a.HW)
                        z1x[(size_t)b * 16 * a.NB1 * a.HW + (((size_t)mg * a.HW + pp) * 4 + (ln >> 4)) * 4 + i] = sum;
                }
                __syncthreads();
            }
        }
        // ---- the barrier among the workgroups of this XCD
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wavefront's z1 stores are in the L2 (and its weight loads have landed)
        __syncthreads();
        TDC_PROBE(3);
        if (pass == 1) break;
        if (wave == 0) {
            const unsigned target = own + 1u;
            if (lane == 0) __hip_atomic_store(my_arrive + role, target, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            unsigned polls = 0;
            bool ok;
            while (true) {
                unsigned v = target;
                if (lane < a.Wn) v = (unsigned)__builtin_amdgcn_raw_buffer_load_b32(ars_flags, lane * 4, 0, 16);   // sc1: misses the L1
                ok = __builtin_amdgcn_ballot_w64((int)(v - target) < 0) == 0;
                if (ok || polls++ >= a.wait_limit) break;
            }
            if (lane == 0) {
                go = ok ? 1 : 0;
                if (!ok) atomicAdd(a.arrive + 8 * 32, 1u);   // counted, for the curious
            }
        }
        __syncthreads();
        if (go) break;
        // The others did not all arrive within the wait: their workgroups may not be resident yet (other streams' kernels
        // hold the compute units), and a workgroup that spins for them keeps its own compute unit from them.  So it stops
        // waiting and computes every stage-1 unit itself, into the same copy of z1: the values are bit-identical to what
        // the others write or will write (same teams, same order of sums), so concurrent writers and readers of a cell
        // see one and the same value.  Slow (all of stage 1 on one workgroup) and never a deadlock.
        role1 = 0; wn1 = 1; rounds1 = (a.n1 + teams - 1) / teams;
    }
    TDC_PROBE(4);

    // ---- the merged K x K GEMM R1 -> N on this XCD's z1
    {
        const int tw = tw2, teams = teams2, team = team2, wt = wt2;
        const int rounds = NK > 0 ? 1 : a.rounds2;
        for (int r = 0; r < rounds; ++r) {
            int b, mg, pg;
            bool live;
            tdc_f4 acc[1][1];
            if (NK > 0) {
                b = b2; mg = mg2; pg = pg2; live = live2;
                const tdc_rsrc zrs = tdc_make_rsrc(z1x + (size_t)b * 16 * a.NB1 * a.HW, (unsigned)(16 * a.NB1) * a.HW * 4u);
                const bool pval = 16 * pg + l16 < a.P;
                const int poff = ih2 * a.W + iw2;
                tdc_f4 zk[NK > 0 ? NK : 1];
                int dg = dg0, rr = r0, ss = s0;
#pragma unroll
                for (int k = 0; k < NK; ++k) {
                    const int h = ih2 + rr, w = iw2 + ss;
                    const bool ok = pval && k < cnt2 && h >= 0 && h < a.H && w >= 0 && w < a.W;
                    zk[k] = tdc_buf_load4(zrs, ((unsigned)((dg * a.HW + poff + rr * a.W + ss) * 16 + 4 * g) * 4u) | (ok ? 0u : TDC_OOB));
                    if (++dg == a.NB1) {
                        dg = 0;
                        if (++ss == a.K) {
                            ss = 0;
                            ++rr;
                        }
                    }
                }
                TDC_PROBE(5);
                acc[0][0] = tdc_f4_zero();
#pragma unroll
                for (int k = 0; k < NK; ++k)
                    if (k < cnt2) {
                        const tdc_f4 av[1] = {wk[k]}, bv[1] = {zk[k]};
                        tdc_mma_group<1, 1>(acc, av, bv);
                    }
            } else {
                const int u = (r * G + lw) * teams + team;
                live = u < a.n2;
                const int bm = tdc_div(live ? u : 0, a.div_npb2);
                pg = (live ? u : 0) - bm * a.npb2;   // (b, channel block), pixel group
                b = tdc_div(bm, a.div_NB3);
                mg = bm - b * a.NB3;
                GemmNext<2, TDC_ACT_BLOCKED, 1, 1> next;
                next.wstride = 0;
                next.wrs = tdc_make_rsrc(a.wm_p + (size_t)mg * a.KG2 * 256, (unsigned)a.KG2 * 1024u);
                next.ars = tdc_make_rsrc(z1x + (size_t)b * 16 * a.NB1 * a.HW, (unsigned)(16 * a.NB1) * a.HW * 4u);
                next.wlane = lane * 16u;
                next.act_pix = a.HW; next.C = 16 * a.NB1; next.NBk = a.NB1; next.K = a.K; next.H = a.H; next.W = a.W; next.g = g;
                const int p = 16 * pg + l16;
                next.pval[0] = p < a.P;
                {
                    const int i = tdc_div(p, a.div_Wo), j = p - i * a.Wo;
                    next.ih0[0] = i * a.stride - a.pad;
                    next.iw0[0] = j * a.stride - a.pad;
                    next.poff[0] = next.ih0[0] * a.W + next.iw0[0];
                }
                next.kg = kg02;
                next.kg_end = live ? kg02 + q2 + (wt < rem2 ? 1 : 0) : kg02;
                next.dg = dg0; next.r = r0; next.s = s0;
                TdcPipe<1, 1, U> pipe;
                pipe.start(next);
                TDC_PROBE(5);
                pipe.run(acc, next.kg_end - kg02, next);
            }
            TDC_PROBE(6);
            const int p = 16 * pg + l16;
            float *__restrict__ yb = a.y + (size_t)b * a.N * a.P;
            if (tw == 1) {
                if (live && p < a.P) {
                    if (a.nhwc) {
                        const int m = 16 * mg + 4 * g;
                        if (m < a.N) tdc_store_nhwc(a.y, a.epi, acc[0][0], m, ((size_t)b * a.P + p) * a.N + m);
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int m = 16 * mg + 4 * g + i;
                            if (m < a.N) {
                                const size_t idx = (size_t)m * a.P + p;
                                yb[idx] = tdc_apply_epilogue(a.epi, acc[0][0][i], m, (size_t)b * a.N * a.P + idx);
                            }
                        }
                    }
                }
                continue;
            }
            if (a.nhwc) {
                red4[wave * 64 + lane] = acc[0][0];
                __syncthreads();
                for (int e = wt * 64 + lane; e < 256; e += tw * 64) {
                    float sum = red[team * tw * 256 + e];
                    for (int ww = 1; ww < tw; ++ww) sum += red[(team * tw + ww) * 256 + e];
                    const int i = e & 3, ln = (e >> 2) & 63;
                    const int pp = 16 * pg + (ln & 15), m = 16 * mg + 4 * (ln >> 4) + i;
                    if (live && pp < a.P && m < a.N) {
                        const size_t idx = ((size_t)b * a.P + pp) * a.N + m;
                        a.y[idx] = tdc_apply_epilogue(a.epi, sum, m, idx);
                    }
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) red[wave * 256 + i * 64 + lane] = acc[0][0][i];
                __syncthreads();
                for (int e = wt * 64 + lane; e < 256; e += tw * 64) {
                    float sum = red[team * tw * 256 + e];
                    for (int ww = 1; ww < tw; ++ww) sum += red[(team * tw + ww) * 256 + e];
                    const int ln = e & 63, i = e >> 6;
                    const int pp = 16 * pg + (ln & 15), m = 16 * mg + 4 * (ln >> 4) + i;
                    if (live && pp < a.P && m < a.N) {
                        const size_t idx = (size_t)m * a.P + pp;
                        yb[idx] = tdc_apply_epilogue(a.epi, sum, m, (size_t)b * a.N * a.P + idx);
                    }
                }
            }
            __syncthreads();
        }
    }
    TDC_PROBE(7);
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

// MERGED_XCD: see tdc_merged_xcd_kernel.  `waves[0]`, `waves[1]`: wavefronts that split the contraction of one
// stage-1 / one merged-GEMM unit (1, 2, 4 or 8; a workgroup always has 8 wavefronts).
bool tdc_merged_xcd_supported(const tdc_tuning &t)
{
    for (int i = 0; i < 2; ++i) {
        const int w = t.waves[i];
        if (!(w == 1 || w == 2 || w == 4 || w == 8) || t.mb[i] != 1 || t.pb[i] != 1) return false;
    }
    return true;
}

int tdc_merged_xcd_grid(const TdcDims &d, const tdc_tuning &t)
{
    const long n1 = (long)d.B * d.NB1 * ((d.H * d.W + 15) / 16), n2 = (long)d.B * d.NB3 * ((d.Ho * d.Wo + 15) / 16);
    const long teams1 = 8 / t.waves[0], teams2 = 8 / t.waves[1];
    long wn = std::max((n1 + teams1 - 1) / teams1, (n2 + 8 * teams2 - 1) / (8 * teams2));
    wn = std::min(32L, std::max(1L, wn));
    return (int)(8 * wn);
}

hipError_t tdc_launch_merged_xcd(const TdcDims &d, const tdc_tuning &t, hipStream_t s, const float *x, const float *uin_p,
                                 const float *wm_p, float *z1c, unsigned *arrive, unsigned *status, unsigned wait_limit,
                                 float *y, const TdcEpi &epi)
{
    XcdArgs a;
    a.x = x; a.uin_p = uin_p; a.wm_p = wm_p; a.z1c = z1c; a.y = y; a.arrive = arrive; a.status = status; a.epi = epi;
    a.HW = d.H * d.W; a.P = d.Ho * d.Wo;
    a.z1_stride = (unsigned)((size_t)d.B * 16 * d.NB1 * a.HW);
    a.wait_limit = wait_limit;
    a.C = d.C; a.N = d.N; a.NB1 = d.NB1; a.NB3 = d.NB3; a.KG1 = d.KG1; a.KG2 = d.K * d.K * d.NB1;
    a.H = d.H; a.W = d.W; a.Wo = d.Wo; a.K = d.K; a.stride = d.stride; a.pad = d.pad;
    const int tw1 = t.waves[0], tw2 = t.waves[1];
    a.lg1 = tw1 == 8 ? 3 : tw1 == 4 ? 2 : tw1 == 2 ? 1 : 0;
    a.lg2 = tw2 == 8 ? 3 : tw2 == 4 ? 2 : tw2 == 2 ? 1 : 0;
    a.q1 = a.KG1 / tw1; a.rem1 = a.KG1 % tw1; a.q2 = a.KG2 / tw2; a.rem2 = a.KG2 % tw2;
    a.npb1 = (a.HW + 15) / 16; a.npb2 = (a.P + 15) / 16;
    a.n1 = d.B * d.NB1 * a.npb1; a.n2 = d.B * d.NB3 * a.npb2;
    const int G = tdc_merged_xcd_grid(d, t);
    a.Wn = G / 8;
    const int teams1 = 8 / tw1, teams2 = 8 / tw2;
    a.rounds1 = (a.n1 + a.Wn * teams1 - 1) / (a.Wn * teams1);
    a.rounds2 = (a.n2 + G * teams2 - 1) / (G * teams2);
    a.nhwc = d.nhwc;
    a.div_Wo = tdc_make_div((unsigned)d.Wo); a.div_NBk = tdc_make_div((unsigned)d.NB1); a.div_K = tdc_make_div((unsigned)d.K);
    a.div_npb1 = tdc_make_div((unsigned)a.npb1); a.div_npb2 = tdc_make_div((unsigned)a.npb2);
    a.div_NB1 = tdc_make_div((unsigned)d.NB1); a.div_NB3 = tdc_make_div((unsigned)d.NB3);
    // weight fragments held in registers across the barrier: when the merged GEMM is one pass of at most 10 k-groups
    // per wavefront (compiled sizes 3, 5, 7, 10)
    const int kpw = (a.KG2 + tw2 - 1) / tw2;
    const int nk = a.rounds2 > 1 || kpw > 10 ? 0 : kpw <= 3 ? 3 : kpw <= 5 ? 5 : kpw <= 7 ? 7 : 10;
#define TDC_CASE(N_)                                                                                            \
    if (nk == N_) {                                                                                             \
        if (d.nhwc) hipLaunchKernelGGL((tdc_merged_xcd_kernel<TDC_ACT_NHWC, N_>), dim3(G), dim3(512), 0, s, a); \
        else hipLaunchKernelGGL((tdc_merged_xcd_kernel<TDC_ACT_NCHW, N_>), dim3(G), dim3(512), 0, s, a);        \
        return hipGetLastError();                                                                               \
    }
    TDC_CASE(0) TDC_CASE(3) TDC_CASE(5) TDC_CASE(7) TDC_CASE(10)
#undef TDC_CASE
    return hipErrorInvalidValue;
}

// Can `grid` workgroups of the kernel be resident on the current device at once?
hipError_t tdc_merged_xcd_resident(int grid, bool nhwc, bool *fits)
{
    int dev = 0, cus = 0, per_cu = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess)
        // the instance with the most registers stands for all
        e = nhwc ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, tdc_merged_xcd_kernel<TDC_ACT_NHWC, 10>, 512, 0)
                 : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, tdc_merged_xcd_kernel<TDC_ACT_NCHW, 10>, 512, 0);
    // every XCD must hold its eighth of the grid on its own compute units
    *fits = e == hipSuccess && cus % 8 == 0 && (long)(grid / 8) <= (long)(cus / 8) * per_cu;
    return e;
}
