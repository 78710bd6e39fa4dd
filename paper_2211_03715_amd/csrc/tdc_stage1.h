// Stage 1 (Eq. 2) of the one-launch kernels: the z1 tile of a workgroup, U_in^T x for every pixel
// of its input tile (halo included), straight from global memory into MFMA operands and on into
// LDS cells.
//
// The tile's 16-pixel blocks and the 16-channel blocks of R1 are grouped into MB1 x PB register
// tiles ("units") dealt round-robin to the wavefronts, the channel groups of one pixel group next to
// each other: wavefronts that need the same pixels of x load them at the same time, so x comes from
// HBM once however many channel groups there are.  A wavefront treats ALL its units as one
// stream of k-groups: operands travel in two register buffers of U k-groups, the loads of one
// buffer are issued before the MFMAs of the other, and the stream runs on across unit
// boundaries -- the first operands of the next unit are already in flight while the last
// k-groups of the current one are multiplied.  (Restarting the pipeline per unit exposes one full
// memory latency per unit, which is what bounds this stage once a wavefront has several units,
// i.e. in the throughput regime.)  A unit occupies ceil(KG1 / U) buffers; k-groups past KG1 and
// units past the last one fetch nothing (address steering, see tdc_mfma.h) and multiply zeros.
#ifndef TDC_STAGE1_H
#define TDC_STAGE1_H

#include "tdc_mfma.h"

struct TdcS1Geom {
    const float *x_img;     // this image's activations
    const float *uin_p;     // packed U_in [NB1][KG1] fragments
    int C, H, W, KG1, NB1;
    int QB, Q, QW;          // input tile: 16-pixel blocks, pixels, row length
    int h0, w0;             // image coordinates of the tile's first pixel (may be negative)
    int pitch1;             // z1 tile row pitch in LDS, in cells
    TdcDiv div_QW;
    unsigned inv_mg;        // ceil(2^20 / (NB1 / MB1)), from the host: unit u = pixel group (u * inv_mg) >> 20, channel group the rest
    // run-major form (TdcStage1R): tile rows, aligned 4-pixel runs per row, 64-pixel blocks of runs
    int QH, RPR, n_sb;
    TdcDiv div_RPR;
};

template <int MB1, int PB, int U, bool NHWC>
struct TdcStage1 {
    const TdcS1Geom &s;
    tdc_rsrc xrs, urs;
    int lane, g, l16, wave, nw;
    int n_pg, n_units;
    unsigned n_mg, inv_mg;  // channel groups and the multiplier that divides by them
    // fetch-side cursor: unit, k-group slot within the unit (dead at and beyond KG1), its channel group
    int fu, fkg, fmg, slots;
    unsigned xoff[PB];      // byte offset of this lane's pixel (NCHW: within a channel row), or TDC_OOB
    tdc_f4 a0[U][MB1], a1[U][MB1], b0[U][PB], b1[U][PB];

    __device__ __forceinline__ TdcStage1(const TdcS1Geom &geom, int lane_, int wave_, int nw_) : s(geom)
    {
        lane = lane_; g = lane_ >> 4; l16 = lane_ & 15; wave = wave_; nw = nw_;
        const int HW = s.H * s.W;
        xrs = tdc_make_rsrc(s.x_img, (unsigned)s.C * HW * 4u);
        urs = tdc_make_rsrc(s.uin_p, (unsigned)s.NB1 * s.KG1 * 1024u);
        n_pg = (s.QB + PB - 1) / PB;
        n_mg = (unsigned)(s.NB1 / MB1);
        n_units = n_pg * (int)n_mg;
        inv_mg = s.inv_mg;
        slots = (s.KG1 + U - 1) / U * U;
        fu = wave;
        place();
    }

    // operand addresses of unit fu
    __device__ __forceinline__ void place()
    {
        fkg = 0;
        const bool live = fu < n_units;
        const int pg = live ? (int)(((unsigned)fu * inv_mg) >> 20) : 0;
        fmg = live ? fu - pg * (int)n_mg : 0;
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
            const int q = 16 * (pg * PB + pb) + l16;
            const int qh = tdc_div(q, s.div_QW), qw = q - qh * s.QW;
            const int h = s.h0 + qh, w = s.w0 + qw;
            const bool ok = live && q < s.Q && h >= 0 && h < s.H && w >= 0 && w < s.W;
            xoff[pb] = ok ? (unsigned)(h * s.W + w) * (NHWC ? 4u * s.C : 4u) : TDC_OOB;
        }
    }

    __device__ __forceinline__ void fetch_group(tdc_f4 (&av)[MB1], tdc_f4 (&bv)[PB])
    {
        const unsigned dead = (fkg < s.KG1 && fu < n_units) ? 0u : TDC_OOB;
#pragma unroll
        for (int mb = 0; mb < MB1; ++mb)
            av[mb] = tdc_buf_load4(urs, ((unsigned)((fmg * MB1 + mb) * s.KG1 + fkg) * 1024u + lane * 16u) | dead);
        if (NHWC) {
            const int c = 16 * fkg + 4 * g;
            const unsigned cbad = c < s.C ? dead : TDC_OOB;
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) bv[pb] = tdc_buf_load4(xrs, (xoff[pb] + 4u * c) | cbad | (xoff[pb] & TDC_OOB));
        } else {
            // channels past C lie beyond the descriptor and read as 0 by themselves
            const unsigned HW4 = (unsigned)(s.H * s.W) * 4u;
            const unsigned c0 = (unsigned)(16 * fkg + 4 * g) * HW4;
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) {
                const unsigned o = (c0 + xoff[pb]) | dead | (xoff[pb] & TDC_OOB);
                bv[pb] = (tdc_f4){tdc_buf_load(xrs, o), tdc_buf_load(xrs, o + HW4), tdc_buf_load(xrs, o + 2u * HW4),
                                  tdc_buf_load(xrs, o + 3u * HW4)};
            }
        }
        if (++fkg == slots) {
            fu += nw;
            place();
        }
    }

    __device__ __forceinline__ void fetch0()
    {
#pragma unroll
        for (int u = 0; u < U; ++u) fetch_group(a0[u], b0[u]);
    }
    __device__ __forceinline__ void fetch1()
    {
#pragma unroll
        for (int u = 0; u < U; ++u) fetch_group(a1[u], b1[u]);
    }

    // Issue the loads of the wavefront's first buffer; call well ahead of run().
    __device__ __forceinline__ void prefetch() { fetch0(); }
    // every cell of the tile is produced by a unit (pixels outside the image read x = 0)
    __device__ __forceinline__ void zero_outside(tdc_f4 *) const {}

    // All units of this wavefront; the finished z1 blocks go to their LDS cells.
    __device__ __forceinline__ void run(tdc_f4 *__restrict__ z1s)
    {
        const int spu = slots / U;       // buffers per unit
        const int mine = wave < n_units ? (n_units - wave + nw - 1) / nw : 0;
        const int total = mine * spu;
        int cu = wave, cb = 0;           // compute-side cursor: unit and buffer within it
        tdc_f4 acc[MB1][PB];
        const auto clear = [&]() {
#pragma unroll
            for (int mb = 0; mb < MB1; ++mb)
#pragma unroll
                for (int pb = 0; pb < PB; ++pb) acc[mb][pb] = tdc_f4_zero();
        };
        const auto finish_buffer = [&]() {
            if (++cb < spu) return;
            const int pg = (int)(((unsigned)cu * inv_mg) >> 20), mg = cu - pg * (int)n_mg;
#pragma unroll
            for (int mb = 0; mb < MB1; ++mb)
#pragma unroll
                for (int pb = 0; pb < PB; ++pb)
                    if (pg * PB + pb < s.QB)
                        z1s[((mg * MB1 + mb) * 4 + g) * s.pitch1 + 16 * (pg * PB + pb) + l16] = acc[mb][pb];
            cu += nw;
            cb = 0;
            clear();
        };
        clear();
        for (int i = 0; i < total; i += 2) {
            fetch1();
#pragma unroll
            for (int u = 0; u < U; ++u) tdc_mma_group<MB1, PB>(acc, a0[u], b0[u]);
            finish_buffer();
            fetch0();
            if (i + 1 < total) {
#pragma unroll
                for (int u = 0; u < U; ++u) tdc_mma_group<MB1, PB>(acc, a1[u], b1[u]);
                finish_buffer();
            }
        }
    }
};

// Stage 1 for NCHW activations with 16-byte loads ("run-major").  In NCHW a lane's four B-operand
// values of the form above are four channels of one pixel, 4 bytes each at channel stride: many
// small requests, partly used cache lines.  Here a lane owns a RUN of four consecutive pixels of a
// tile row instead, aligned to 4 in image coordinates (the image width is a multiple of 4, so a run
// is inside the image or outside it as a whole), and loads it with one 16-byte load per channel:
//   lane (g, l16), k-group kg, q = 0..3:  b[q] = x[channel 16*kg + 4*q + g][run l16, pixels 0..3]
// The four MFMAs of (q, t) contract over the four channels 4*q + g and accumulate pixel t of the run
// into accumulator t, so a unit is 16 runs = 64 pixels and four accumulators per channel block; the
// U_in fragments come re-laid-out with the matching k order (lane (g, l16), component q = channel
// 16*kg + 4*q + g).  The accumulator of (channel block, t) is, per lane, the z1 cell of pixel t of the
// lane's run; cells of tile columns that lie outside the image are never produced by a run and are
// zeroed by zero_outside() instead.
template <int MB1, int U>
struct TdcStage1R {
    const TdcS1Geom &s;
    tdc_rsrc xrs, urs;
    int lane, g, l16, wave, nw;
    int n_units, wa;        // wa: image column of the first run of a row (a multiple of 4, >= 0)
    unsigned n_mg, inv_mg;  // channel groups and the multiplier that divides by them
    int fu, fkg, fmg, slots;
    unsigned xoff;          // byte offset of this lane's run within a channel plane, or TDC_OOB
    tdc_f4 a0[U][MB1], a1[U][MB1], b0[U][4], b1[U][4];

    __device__ __forceinline__ TdcStage1R(const TdcS1Geom &geom, int lane_, int wave_, int nw_) : s(geom)
    {
        lane = lane_; g = lane_ >> 4; l16 = lane_ & 15; wave = wave_; nw = nw_;
        const int HW = s.H * s.W;
        xrs = tdc_make_rsrc(s.x_img, (unsigned)s.C * HW * 4u);
        urs = tdc_make_rsrc(s.uin_p, (unsigned)s.NB1 * s.KG1 * 1024u);
        n_mg = (unsigned)(s.NB1 / MB1);
        n_units = s.n_sb * (int)n_mg;
        inv_mg = s.inv_mg;
        slots = (s.KG1 + U - 1) / U * U;
        wa = s.w0 > 0 ? (s.w0 & ~3) : 0;
        fu = wave;
        place();
    }

    // Tile cells whose image column is outside [0, W): all rows, all channel planes.  Disjoint from
    // what the runs write, so no barrier is needed between the two.
    __device__ __forceinline__ void zero_outside(tdc_f4 *__restrict__ z1s) const
    {
        const int left = s.w0 < 0 ? -s.w0 : 0;                               // columns qw < left
        const int right = max(s.w0 + s.QW - s.W, 0);                          // columns qw >= QW - right
        const int per_row = left + right, planes = 4 * s.NB1;
        const int total = per_row * s.QH * planes;
        for (int e = 64 * wave + lane; e < total; e += 64 * nw) {
            const int c = e % per_row, r = (e / per_row) % s.QH, pl = e / (per_row * s.QH);
            const int qw = c < left ? c : s.QW - right + (c - left);
            z1s[pl * s.pitch1 + r * s.QW + qw] = tdc_f4_zero();
        }
    }

    __device__ __forceinline__ void place()
    {
        fkg = 0;
        const bool live = fu < n_units;
        const int sb = live ? (int)(((unsigned)fu * inv_mg) >> 20) : 0;
        fmg = live ? fu - sb * (int)n_mg : 0;
        const int rho = 16 * sb + l16;
        const int qh = tdc_div(rho, s.div_RPR), rc = rho - qh * s.RPR;
        const int h = s.h0 + qh, col = wa + 4 * rc;
        const bool ok = live && qh < s.QH && h >= 0 && h < s.H && col < s.W;
        xoff = ok ? (unsigned)(h * s.W + col) * 4u : TDC_OOB;
    }

    __device__ __forceinline__ void fetch_group(tdc_f4 (&av)[MB1], tdc_f4 (&bv)[4])
    {
        const unsigned dead = (fkg < s.KG1 && fu < n_units) ? 0u : TDC_OOB;
#pragma unroll
        for (int mb = 0; mb < MB1; ++mb)
            av[mb] = tdc_buf_load4(urs, ((unsigned)((fmg * MB1 + mb) * s.KG1 + fkg) * 1024u + lane * 16u) | dead);
        // channels past C lie beyond the descriptor and read as 0 by themselves
        const unsigned HW4 = (unsigned)(s.H * s.W) * 4u;
        const unsigned o = ((unsigned)(16 * fkg + g) * HW4 + xoff) | dead | (xoff & TDC_OOB);
#pragma unroll
        for (int q = 0; q < 4; ++q) bv[q] = tdc_buf_load4(xrs, o + (unsigned)(4 * q) * HW4);
        if (++fkg == slots) {
            fu += nw;
            place();
        }
    }

    __device__ __forceinline__ void fetch0()
    {
#pragma unroll
        for (int u = 0; u < U; ++u) fetch_group(a0[u], b0[u]);
    }
    __device__ __forceinline__ void fetch1()
    {
#pragma unroll
        for (int u = 0; u < U; ++u) fetch_group(a1[u], b1[u]);
    }
    __device__ __forceinline__ void prefetch() { fetch0(); }

    __device__ __forceinline__ void run(tdc_f4 *__restrict__ z1s)
    {
        const int spu = slots / U;
        const int mine = wave < n_units ? (n_units - wave + nw - 1) / nw : 0;
        const int total = mine * spu;
        int cu = wave, cb = 0;
        tdc_f4 acc[MB1][4];
        const auto clear = [&]() {
#pragma unroll
            for (int mb = 0; mb < MB1; ++mb)
#pragma unroll
                for (int t = 0; t < 4; ++t) acc[mb][t] = tdc_f4_zero();
        };
        const auto mma = [&](const tdc_f4 (&av)[MB1], const tdc_f4 (&bv)[4]) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int t = 0; t < 4; ++t)
#pragma unroll
                    for (int mb = 0; mb < MB1; ++mb) acc[mb][t] = tdc_mfma(av[mb][q], bv[q][t], acc[mb][t]);
        };
        const auto finish_buffer = [&]() {
            if (++cb < spu) return;
            const int sb = (int)(((unsigned)cu * inv_mg) >> 20), mg = cu - sb * (int)n_mg;
            const int rho = 16 * sb + l16;
            const int qh = tdc_div(rho, s.div_RPR), rc = rho - qh * s.RPR;
            const int qw0 = wa + 4 * rc - s.w0;            // tile column of the run's first pixel (may be < 0)
            if (qh < s.QH) {
#pragma unroll
                for (int mb = 0; mb < MB1; ++mb)
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        if (qw0 + t >= 0 && qw0 + t < s.QW)
                            z1s[((mg * MB1 + mb) * 4 + g) * s.pitch1 + qh * s.QW + qw0 + t] = acc[mb][t];
            }
            cu += nw;
            cb = 0;
            clear();
        };
        clear();
        for (int i = 0; i < total; i += 2) {
            fetch1();
#pragma unroll
            for (int u = 0; u < U; ++u) mma(a0[u], b0[u]);
            finish_buffer();
            fetch0();
            if (i + 1 < total) {
#pragma unroll
                for (int u = 0; u < U; ++u) mma(a1[u], b1[u]);
                finish_buffer();
            }
        }
    }
};

// Copy of the packed core and U_out arrays (adjacent in LDS) into LDS, CH 16-byte pieces per thread
// and round.  load() and store() are separate so that the first round's loads can be issued before
// stage 1 and stored after it: they then travel while stage 1 computes.
template <int CH>
struct TdcWeightCopy {
    tdc_f4 tmp[CH];
    __device__ __forceinline__ void load(const tdc_f4 *__restrict__ core4, int n_core, const tdc_f4 *__restrict__ uout4,
                                         int n_uout, int base)
    {
        const int n = n_core + n_uout;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int i = min(base + (int)threadIdx.x + c * (int)blockDim.x, n - 1);
            const tdc_f4 *__restrict__ src = i < n_core ? core4 + i : uout4 + (i - n_core);
            tmp[c] = *src;
        }
    }
    __device__ __forceinline__ void store(tdc_f4 *__restrict__ dst, int n, int base) const
    {
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int i = base + (int)threadIdx.x + c * (int)blockDim.x;
            if (i < n) dst[i] = tmp[c];
        }
    }
};

// Layouts a one-launch kernel is compiled for: how x is read and y is written.
enum { TDC_LAY_NCHW = 0, TDC_LAY_NHWC = 1, TDC_LAY_NCHW_RUNS = 2 };   // RUNS: NCHW with the run-major stage 1

#endif
