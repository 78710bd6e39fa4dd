// Device helpers around v_mfma_f32_16x16x4_f32 (gfx950), shared by the GEMM and fused kernels.
//
// Operand layout of one step D += A*B with A 16x4, B 4x16, D 16x16, 64 lanes:
//   A : lane l holds A[m = l%16][k = l/16]
//   B : lane l holds B[k = l/16][p = l%16]
//   D : lane l holds D[m = 4*(l/16) + i][p = l%16] in register i = 0..3
// Here m is an output channel, p a pixel and k the contraction index, so pixels run
// along the lanes: activation loads and stores are contiguous in NCHW.
//
// A "k-group" is 16 consecutive contraction indices = four MFMA steps j = 0..3.  Within a
// k-group, step j of lane group g = l/16 consumes contraction index 4*g + j.  With this
// order the four accumulator registers a lane holds after one stage (channels 4*g + i of a
// 16-channel block, i = 0..3) are exactly the four B operands the same lane position needs
// for that block in the next stage, so an intermediate tile moves through LDS as one
// 16-byte write and one 16-byte read per lane and k-group.
#ifndef TDC_MFMA_H
#define TDC_MFMA_H

#include <hip/hip_runtime.h>

#include "tdc_internal.h"
#include "tdc_div.h"

typedef float tdc_f4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ tdc_f4 tdc_mfma(float a, float b, tdc_f4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ tdc_f4 tdc_f4_zero() { return (tdc_f4){0.f, 0.f, 0.f, 0.f}; }

// Global operands are fetched with buffer loads: the hardware range check returns 0 for an
// offset at or beyond the descriptor's size, so a lane that must read "nothing" (a pixel outside
// the image or the tile, a channel past C, a k-group past the end of the range) just gets the
// bit TDC_OOB set in its byte offset.  No branch and, unlike a select on the loaded value,
// no wait for the load at the point of issue: loads can stay in flight across the MFMAs of the
// other register buffer.  Descriptors cover less than 2 GiB.
typedef __amdgpu_buffer_rsrc_t tdc_rsrc;
constexpr unsigned TDC_OOB = 0x80000000u;

__device__ __forceinline__ tdc_rsrc tdc_make_rsrc(const void *base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

__device__ __forceinline__ float tdc_buf_load(tdc_rsrc r, unsigned byte_off)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)byte_off, 0, 0));
}

__device__ __forceinline__ tdc_f4 tdc_buf_load4(tdc_rsrc r, unsigned byte_off)
{
    typedef unsigned u4 __attribute__((ext_vector_type(4)));
    return __builtin_bit_cast(tdc_f4, (u4)__builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, 0));
}

// The optional epilogue on one output value: channel n, element index idx within y.  The branches
// are wave-uniform; without an epilogue nothing is loaded.
__device__ __forceinline__ float tdc_apply_epilogue(const TdcEpi &e, float v, int n, size_t idx)
{
    if (e.bias) v += e.bias[n];
    if (e.residual) v += e.residual[idx];
    return e.relu ? fmaxf(v, 0.f) : v;
}

// NHWC output: the four accumulator registers of a lane are channels n .. n+3 (n a multiple of 4)
// of one pixel, i.e. 16 contiguous bytes of y.  `cell` is the element index of channel n of that
// pixel within the whole tensor; y and the residual are 16-byte aligned.
// STREAM: store with the non-temporal hint (see tdc_store4_stream).
template <bool STREAM = false>
__device__ __forceinline__ void tdc_store_nhwc(float *__restrict__ y, const TdcEpi &e, tdc_f4 v, int n, size_t cell)
{
    if (e.bias) v += (tdc_f4){e.bias[n], e.bias[n + 1], e.bias[n + 2], e.bias[n + 3]};
    if (e.residual) v += *reinterpret_cast<const tdc_f4 *>(e.residual + cell);
    if (e.relu) v = (tdc_f4){fmaxf(v[0], 0.f), fmaxf(v[1], 0.f), fmaxf(v[2], 0.f), fmaxf(v[3], 0.f)};
    if (STREAM) __builtin_nontemporal_store(v, reinterpret_cast<tdc_f4 *>(y + cell));
    else *reinterpret_cast<tdc_f4 *>(y + cell) = v;
}

// A 16-byte store with the non-temporal hint: the line leaves the L2 early instead of waiting there, dirty, for the
// write-back at the end of the kernel.  For the throughput kernels' NHWC outputs (whole 16-byte cells of consecutive
// channels, tens of MB per call) this took 4-8 % off the call: the write-back no longer sits between one launch and
// the next.  Not for NCHW outputs, whose 16-byte pieces of many channel planes rely on the L2 to be merged into
// lines (measured up to 1.8x slower at batch 128), nor for the small outputs of the latency kernels.
__device__ __forceinline__ void tdc_store4_stream(tdc_f4 *p, tdc_f4 v) { __builtin_nontemporal_store(v, p); }

// Kernel arguments arrive through scalar loads that the compiler issues where a value is first needed.  A
// prologue that needs some arguments for its tile arithmetic and others (the pointers, the block size) for
// its first vector load then makes two or three DEPENDENT scalar-memory round trips before that load -- at
// kernel durations of a few microseconds a measurable part of the whole.  TDC_FETCH_NOW(outs, ins) is one
// empty asm statement: `ins` ("s"(x), "s"(y), ...) are the arguments the prologue will need, which must all
// be in scalar registers at that one point; `outs` ("+s"(v), ...) are a few values that everything in the
// prologue is computed from (block size, grid size, the first divisor), passed through the statement so
// that none of that arithmetic can be scheduled in front of it.  All argument loads are then issued together
// at the top of the kernel and cost one round trip.
#define TDC_FETCH_NOW(outs, ...) asm volatile("" : outs : __VA_ARGS__)
#define TDC_OUTS(...) __VA_ARGS__

__device__ __forceinline__ int tdc_div(int x, const TdcDiv &d)
{
    return (int)tdc_div_from_hi((unsigned)x, __umulhi(d.m, (unsigned)x), d);
}

// acc[mb][pb] += A(mb, step j) * B(pb, step j) for the four steps of one k-group.  Successive
// MFMAs may target the same accumulator: v_mfma_f32_16x16x4_f32 issues every 32 cycles even in a
// dependent chain (measured), so no extra accumulators are needed to keep the pipe busy.
template <int MB, int PB>
__device__ __forceinline__ void tdc_mma_group(tdc_f4 (&acc)[MB][PB], const tdc_f4 (&a)[MB], const tdc_f4 (&b)[PB])
{
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) acc[mb][pb] = tdc_mfma(a[mb][j], b[pb][j], acc[mb][pb]);
}

// Software pipeline over the k-groups of one register tile.  `next(a, b)` fetches the operands
// of the following k-group each time it is called; it is called more often than there are
// k-groups and must then return A = 0 without touching memory out of bounds (by steering the
// address, never by post-processing the loaded value), which keeps the loop body free of
// branches and of waits.  Operands travel in two
// register buffers of U k-groups; the loads of one buffer are issued before the MFMAs of the
// other, so a tile with at most 2*U k-groups waits for memory once.  start() may be called
// well ahead of run() to overlap the first fetch with other work.  run() overwrites acc.
template <int MB, int PB, int U>
struct TdcPipe {
    tdc_f4 a0[U][MB], a1[U][MB];
    tdc_f4 b0[U][PB], b1[U][PB];

    template <class Next>
    __device__ __forceinline__ void start(Next &next)
    {
#pragma unroll
        for (int u = 0; u < U; ++u) next(a0[u], b0[u]);
    }

    template <class Next>
    __device__ __forceinline__ void run(tdc_f4 (&acc)[MB][PB], int nkg, Next &next)
    {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int pb = 0; pb < PB; ++pb) acc[mb][pb] = tdc_f4_zero();
        for (int kg = 0; kg < nkg; kg += 2 * U) {
#pragma unroll
            for (int u = 0; u < U; ++u) next(a1[u], b1[u]);
#pragma unroll
            for (int u = 0; u < U; ++u) tdc_mma_group<MB, PB>(acc, a0[u], b0[u]);
#pragma unroll
            for (int u = 0; u < U; ++u) next(a0[u], b0[u]);
            if (kg + U < nkg) {
#pragma unroll
                for (int u = 0; u < U; ++u) tdc_mma_group<MB, PB>(acc, a1[u], b1[u]);
            }
        }
    }
};

// Phase timestamps for kernel bring-up: compiled in only with -DTDC_PHASE_TIMING, by the probe build
// (`python -m paper_2211_03715_amd.build --probes`, which puts every source into one translation unit and
// writes libtdc_probe.so; never in the shipped library).  Slot s of wavefront w of workgroup b lands in
// tdc_probe_buf[((b*8+w)*16+s)*2 + {0,1}] as (shader clock, 100 MHz wall clock);
// `python -m paper_2211_03715_amd.probes` reads them back.
#ifdef TDC_PHASE_TIMING
__device__ unsigned long long tdc_probe_buf[2 * 8 * 16 * 4096];
#define TDC_PROBE(slot)                                                                             \
    do {                                                                                            \
        if ((threadIdx.x & 63) == 0 && blockIdx.x < 4096 && blockIdx.y == 0) {                      \
            const size_t o = (((size_t)blockIdx.x * 8 + (threadIdx.x >> 6)) * 16 + (slot)) * 2;     \
            tdc_probe_buf[o] = clock64();                                                           \
            tdc_probe_buf[o + 1] = wall_clock64();                                                  \
        }                                                                                           \
    } while (0)
extern "C" int tdc_debug_read_probes(unsigned long long *host, size_t count)
{
    return hipMemcpyFromSymbol(host, HIP_SYMBOL(tdc_probe_buf), count * sizeof(unsigned long long)) == hipSuccess ? 0 : -1;
}
extern "C" int tdc_debug_clear_probes(void)
{
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(tdc_probe_buf)) != hipSuccess) return -1;
    return hipMemset(p, 0, sizeof(tdc_probe_buf)) == hipSuccess ? 0 : -1;
}
#else
#define TDC_PROBE(slot) do { } while (0)
#endif

#endif
