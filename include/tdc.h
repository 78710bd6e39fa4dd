/*
 * tdc.h -- C ABI of the MI355X (gfx950) Tucker-2 convolution library.
 *
 * One call evaluates one Tucker-2-format convolution layer (paper section 3,
 * "Basics of TKD-based Convolution"): a 1x1 projection C -> R1 with the factor
 * U_in (Eq. 2), a K x K "core" convolution R1 -> R2 on the core tensor (Eq. 3)
 * and a 1x1 expansion R2 -> N with the factor U_out (Eq. 4).  The result equals
 * the dense convolution with the kernel of Eq. 1,
 *   K(c,n,r,s) = sum_{d1,d2} core(d1,d2,r,s) * U_in(c,d1) * U_out(d2,n),
 * up to fp32 rounding.  R1, R2 are the paper's Tucker ranks D1, D2; K is the
 * paper's stencil size R = S.
 *
 * All tensor arguments are DEVICE pointers to contiguous fp32 arrays, at least
 * 16-byte aligned, resident on the plan's device:
 *   x      [batch][C][H][W]          input (layout 0, NCHW; layout 1: [batch][H][W][C])
 *   U_in   [C][R1]                   U1(c,d1)
 *   core   [R1][R2][K][K]            core(d1,d2,r,s)  (mode 1 contracts with U_in,
 *                                    mode 2 with U_out; cross-correlation, no flip)
 *   U_out  [R2][N]                   U2(d2,n) as Eq. 4 uses it
 *   y      [batch][N][Ho][Wo]        output (layout 1: [batch][Ho][Wo][N]),
 *                                    Ho = floor((H+2*pad-K)/stride)+1
 * Zero padding `pad` and `stride` apply to the core convolution; stage 1 runs on
 * every input pixel.  tdc_conv_tucker2 applies no bias or activation: the layer is
 * linear in x.  The _ex entry points add an optional fused epilogue (see tdc_epilogue).
 *
 * Ownership: the caller owns x, the weights, y and the stream.  The library
 * never frees or reallocates them.  A plan owns its workspace (intermediates
 * and re-laid-out weights) and releases it in tdc_plan_destroy.  y is fully
 * overwritten; x and y must not overlap.  A plan may be used by one stream at
 * a time (its workspace is not re-entrant).
 *
 * Asynchrony: the conv and pack entry points only enqueue work on the given
 * stream (NULL = the default stream) and return; they never synchronise with
 * the host and never allocate, and a conv call with re-laid-out weights enqueues
 * nothing but its kernels, so it may be captured into a HIP graph.
 *
 * Errors: every function returns a tdc_status (0 = success, negative =
 * failure).  Nothing aborts, throws or prints.
 */
#ifndef TDC_H
#define TDC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum tdc_status {
    TDC_OK = 0,
    TDC_ERR_NULL = -1,            /* a required pointer is NULL                               */
    TDC_ERR_BAD_SHAPE = -2,       /* non-positive size, stride < 1, pad < 0, H + 2*pad < K    */
    TDC_ERR_SHAPE_MISMATCH = -3,  /* shape passed to a call differs from the plan's           */
    TDC_ERR_UNSUPPORTED = -4,     /* valid layer outside the supported domain (see below)     */
    TDC_ERR_ALLOC = -5,           /* device or host allocation failed                         */
    TDC_ERR_HIP = -6,             /* a HIP runtime call or a kernel launch failed             */
    TDC_ERR_BAD_TUNING = -7,      /* a forced tuning does not fit the shape or the hardware   */
    TDC_ERR_TOO_LARGE = -8,       /* tdc_conv_tucker2_static: the layer needs more scratch memory than
                                     TDC_STATIC_SCRATCH_BYTES                                  */
    TDC_ERR_NO_CONVERGENCE = -9,  /* tdc_hosvd_tucker2 / tdc_admm_project: an eigen-decomposition did not reach
                                     its tolerance within the sweep limit; outputs are not written             */
    TDC_ERR_WAIT = -10            /* a TDC_VARIANT_MERGED_XCD kernel found itself on a device whose XCD or workgroup
                                     numbering it was not written for and wrote nothing.  Kernels run asynchronously,
                                     so the error is returned by tdc_plan_status and by every LATER tdc_conv_tucker2
                                     call on the plan, which then enqueues nothing                             */
} tdc_status;

/* Layer geometry.  Supported domain: square K in 1..7; stride in 1..4; pad in 0..K-1; any
 * positive batch (at most 65535), C, N, H, W, R1, R2 for which every tensor has fewer than 2^31
 * elements and one image of x or y (channels rounded up to 16) is smaller than 2 GiB; outside it
 * tdc_plan_create returns TDC_ERR_UNSUPPORTED.
 * layout selects how the activations are stored: 0 = NCHW, x[batch][C][H][W] and
 * y[batch][N][Ho][Wo]; 1 = NHWC, x[batch][H][W][C] and y[batch][Ho][Wo][N] (the pixel-major
 * order the paper writes its tensors in, section 3); an epilogue's residual is laid out like y.
 * NHWC moves channels four at a time: C and N must be multiples of 4 and x, y and the residual
 * 16-byte aligned, else TDC_ERR_UNSUPPORTED.  NCHW plans for large batches read rows whose width is
 * a multiple of 4 sixteen bytes at a time and return TDC_ERR_UNSUPPORTED for an x that is not 16-byte
 * aligned.  Weights have one layout, whatever the activations'. */
typedef struct tdc_shape {
    int32_t batch, C, N, H, W;
    int32_t R1, R2, K;
    int32_t stride, pad;
    int32_t layout;               /* 0 = NCHW, 1 = NHWC.  Other values: TDC_ERR_UNSUPPORTED */
} tdc_shape;

/* Kernel families the selector chooses between (section 5.5 of the paper picks tile
 * sizes with an analytical model; the selector here is this library's own). */
enum {
    TDC_VARIANT_AUTO = 0,   /* let the selector decide                                          */
    TDC_VARIANT_NAIVE = 1,  /* three plain fp32 kernels, one thread per output pixel            */
    TDC_VARIANT_SPLIT = 2,  /* three fp32-MFMA GEMM kernels, intermediates z1/z2 in workspace   */
    TDC_VARIANT_FUSED = 3,  /* one fp32-MFMA kernel per spatial tile, z1/z2 kept in LDS         */
    TDC_VARIANT_CHAIN = 4,  /* fused; each wavefront keeps its z2 columns in registers and feeds
                               them straight into stage 3 (throughput regime)                   */
    TDC_VARIANT_MERGED = 6, /* two kernels: stage 1, then ONE K x K implicit GEMM R1 -> N whose kernel
                               core x_2 U_out is formed when the weights are re-laid out.  More MACs
                               than Eqs. 3+4 (K*K*R1*N against K*K*R1*R2 + R2*N per pixel), same
                               result; its output-channel blocks run in parallel, which pays on
                               small images at batch 1 where launches, not FLOPs, set the latency */
    TDC_VARIANT_FUSED_MERGED = 7, /* one kernel: a workgroup computes stage 1 for its pixel tile into LDS
                               and then the merged stage-2/3 convolution for its own group of output
                               channels; workgroups that share a tile recompute stage 1.  Tuning:
                               tile_h, tile_w (at most 64 pixels), waves[0], mb[0] (stage 1), mb[1] =
                               16-channel output blocks per workgroup (must divide waves[0])       */
    TDC_VARIANT_MERGED_XCD = 8, /* MERGED in ONE launch, for small images at batch 1 where the boundary between
                               MERGED's two kernels is a quarter of the layer's time: the workgroups that
                               run on one XCD (they share its L2) compute all of stage 1 into that XCD's own
                               copy of z1, meet at a barrier among themselves, and run their share of the
                               merged K x K GEMM on it.  The wait at the barrier is bounded: a workgroup whose
                               partners do not arrive in time (a launch of up to 256 workgroups is only fully
                               resident when other streams leave it the room) stops waiting and computes all of
                               stage 1 itself -- slower, same bits, never a deadlock.  Tuning: waves[0],
                               waves[1] = wavefronts that split the contraction of one 16x16 output block in
                               stage 1 / in the merged GEMM (1, 2, 4 or 8); mb and pb must be 1.  Workspace:
                               8 copies of z1.  Never chosen by AUTO                                */
    TDC_VARIANT_DENSE = 5   /* not a Tucker kernel: the undecomposed K x K layer as one implicit-GEMM
                               MFMA kernel, for tdc_conv_dense only.  Never chosen by AUTO; a plan
                               made with it ignores R1 and R2                                   */
};

/* Launch parameters.  Zero in any field means "selector's choice".
 *   tile_h, tile_w : output tile of one workgroup            (FUSED, CHAIN)
 *   waves          : wavefronts (of 64 lanes) per workgroup  (SPLIT: per stage; FUSED, CHAIN: waves[0];
 *                    MERGED: [0] for stage 1, [1] for the merged convolution, likewise mb and pb)
 *   mb, pb         : 16-channel and 16-pixel blocks per wavefront register tile, per stage
 *                    (CHAIN uses mb[0] and pb[0]; its stage-2 tile is all of R2 by construction) */
typedef struct tdc_tuning {
    int32_t variant;
    int32_t tile_h, tile_w;
    int32_t waves[3];
    int32_t mb[3];
    int32_t pb[3];
} tdc_tuning;

typedef struct tdc_plan tdc_plan;   /* opaque, library-owned */

/* Validate `shape`, run the selector (or take `forced` when not NULL), and allocate the
 * workspace on `device`.  On success *out holds the plan. */
int tdc_plan_create(tdc_plan **out, const tdc_shape *shape, int device);
int tdc_plan_create_tuned(tdc_plan **out, const tdc_shape *shape, int device, const tdc_tuning *forced);

/* Re-lay the weights out for the kernels, once, into plan-owned memory (the paper's
 * section 5.2 does the same conversion offline).  Later tdc_conv_tucker2 calls that pass
 * these same three pointers use the stored copy; the caller thereby promises not to
 * change the weights in place without calling this again.  Without this call every
 * tdc_conv_tucker2 re-lays the weights out on the stream first (correct, slower).
 * The re-layout is enqueued on `hip_stream`; a conv call that uses the stored copy from ANOTHER stream
 * must be ordered after it by the caller (an event, or a synchronise): the library adds no dependency
 * between streams. */
int tdc_plan_pack_weights(tdc_plan *plan, void *hip_stream,
                          const float *U_in, const float *core, const float *U_out);

/* Enqueue y = TuckerConv(x; U_in, core, U_out) (Eqs. 2-4).  `shape` must equal the plan's. */
int tdc_conv_tucker2(tdc_plan *plan, void *hip_stream,
                     const float *x, const float *U_in, const float *core, const float *U_out,
                     float *y, const tdc_shape *shape);

/* Optional output epilogue for the _ex entry points: with acc the convolution result,
 *     y = acc + bias[n] + residual[same element as y],   then   y = max(y, 0) if relu != 0,
 * applied in the store of y (no extra pass, no extra launch).  It lets a chain of layers with
 * batch-norm folded into the weights and bias, ReLU, and a ResNet shortcut run as one call per
 * layer (the paper's end-to-end models, section 7.3, have such layers between the Tucker
 * convolutions).  bias: device pointer to N floats or NULL.  residual: device pointer to a tensor
 * shaped and laid out like y, or NULL; it must not overlap y.  A NULL epilogue is no epilogue;
 * tdc_conv_tucker2(...) == tdc_conv_tucker2_ex(..., NULL).  Same ownership, asynchrony and error rules
 * as the plain calls. */
typedef struct tdc_epilogue {
    const float *bias;
    const float *residual;
    int32_t relu;
} tdc_epilogue;

int tdc_conv_tucker2_ex(tdc_plan *plan, void *hip_stream,
                        const float *x, const float *U_in, const float *core, const float *U_out,
                        float *y, const tdc_shape *shape, const tdc_epilogue *epilogue);

/* The undecomposed layer, y = K (*) x with the dense kernel W[C][N][K][K] = K(c,n,r,s) of Eq. 1
 * (same index order as `core`, same padding / stride / cross-correlation rule, x and y as above).
 * This is the "original convolution" of the paper's rank selection (section 6): a layer is only
 * decomposed if its Tucker latency t1 beats the original layer's latency t2 by the threshold
 * theta, so a caller building the latency table needs both from the same library.
 * `plan` must have been created by tdc_plan_create_tuned with variant TDC_VARIANT_DENSE (fields
 * mb[1], pb[1], waves[1] may be forced; R1 and R2 of the shape must be positive and are otherwise
 * ignored); on such a plan tdc_conv_tucker2 and tdc_plan_pack_weights return TDC_ERR_BAD_TUNING, and
 * so do the two calls below on any other plan.  tdc_plan_pack_dense stores the re-laid-out copy of W
 * exactly as tdc_plan_pack_weights does for the factors; without it every call re-lays W out first. */
int tdc_plan_pack_dense(tdc_plan *plan, void *hip_stream, const float *W);
int tdc_conv_dense(tdc_plan *plan, void *hip_stream, const float *x, const float *W, float *y,
                   const tdc_shape *shape);
int tdc_conv_dense_ex(tdc_plan *plan, void *hip_stream, const float *x, const float *W, float *y,
                      const tdc_shape *shape, const tdc_epilogue *epilogue);

/* For callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same result as tdc_conv_tucker2 on a plan of variant
 * TDC_VARIANT_SPLIT (three fp32-MFMA GEMM kernels behind the weight re-layout), but without a plan:
 * the re-laid-out weights and the intermediates z1, z2 live in one device array of
 * TDC_STATIC_SCRATCH_BYTES that is part of the library's code object, so every GPU the library
 * runs on holds that much until the process ends.  The call enqueues six kernels on `hip_stream`
 * and returns; it calls no hipMalloc / hipFree and no allocating library routine, and never
 * synchronises.  It runs on the calling thread's CURRENT device, which must be the device of the
 * stream and of all five tensors.
 * Scratch needed, in floats, each term rounded up to a multiple of 64:
 *     16*ceil(R1/16) * 16*ceil(C/16)  +  16*ceil(R2/16) * K*K * 16*ceil(R1/16)  +  16*ceil(N/16) * 16*ceil(R2/16)
 *   + batch * 16*ceil(R1/16) * H*W    +  batch * 16*ceil(R2/16) * Ho*Wo;
 * a layer that needs more returns TDC_ERR_TOO_LARGE and enqueues nothing.  Other errors as for
 * tdc_plan_create and tdc_conv_tucker2 (NHWC: C, N multiples of 4 and 16-byte aligned x, y).
 * All calls on one GPU share the one array, which keeps the last call's contents; every call
 * overwrites what it reads, so nothing carries over, but two calls that may overlap in time on one
 * GPU (different streams, or the same array through two processes' own copies is fine -- each
 * process has its own) race on it: order them on one stream or with events. */
#define TDC_STATIC_SCRATCH_BYTES (32u * 1024u * 1024u)
int tdc_conv_tucker2_static(void *hip_stream,
                            const float *x, const float *U_in, const float *core, const float *U_out,
                            float *y, const tdc_shape *shape);

/* Release the plan and its workspace.  NULL is accepted. */
int tdc_plan_destroy(tdc_plan *plan);

/* Introspection (host only). */
int tdc_plan_get_tuning(const tdc_plan *plan, tdc_tuning *out);          /* what will be launched   */
int tdc_plan_describe(const tdc_plan *plan, char *buf, size_t buf_len);  /* one line of text        */
size_t tdc_plan_workspace_bytes(const tdc_plan *plan);                   /* device bytes owned      */
int tdc_plan_kernel_count(const tdc_plan *plan);                         /* launches per conv call (weights packed) */
/* TDC_OK, or TDC_ERR_WAIT once a kernel of a TDC_VARIANT_MERGED_XCD plan has reported that it cannot run on this
 * device (sticky; reads a word in pinned host memory that the kernel writes, so call it after the stream has been
 * synchronised to learn about the calls enqueued so far).  Always TDC_OK for other variants; TDC_ERR_NULL for a NULL plan. */
int tdc_plan_status(const tdc_plan *plan);
const char *tdc_status_string(int status);                               /* static string           */
int tdc_version(void);

/* The selector by itself (host only, touches no device): fill every zero field of *inout for a
 * device with `compute_units` CUs and `lds_bytes` of LDS per workgroup.  This is the a-priori
 * model tdc_plan_create uses; see tdc_select.cpp for its terms.  A caller that keeps k independent calls
 * in flight on k streams can ask for a tuning for compute_units / k and hand it to tdc_plan_create_tuned:
 * fewer, larger workgroups per call then leave room for the other calls (measured: up to 20 % more
 * throughput at batch 32 than k plans made for the whole chip). */
int tdc_select_tuning(const tdc_shape *shape, int compute_units, int lds_bytes, tdc_tuning *inout);

/* The selector's estimate, opened up for calibration (host only, touches no device).  The estimate of a tuning is a
 * dot product of fitted coefficients with terms computed from the shape and the tuning; this call returns the terms of
 * the fully specified tuning *tuning (every field set, as tdc_plan_get_tuning or tdc_select_tuning return it):
 * terms[0 .. *n_terms), their names (static strings) in names[] when names is not NULL, and in *model (when not NULL)
 * which coefficient table applies: "fused_latency", "fused_throughput", "chain", "fused_merged" or "stage" (the GEMM
 * launches of SPLIT, MERGED and DENSE, summed over the launches of one call).  A least-squares fit of measured
 * latencies against these terms reproduces the tables the library is built with (paper section 5.5 compares its
 * model with exhaustive search the same way).  TDC_ERR_BAD_TUNING for NAIVE / AUTO, TDC_ERR_BAD_SHAPE if max_terms is
 * too small (32 is enough). */
int tdc_model_terms(const tdc_shape *shape, const tdc_tuning *tuning, int compute_units, int lds_bytes,
                    double *terms, const char **names, int max_terms, int *n_terms, const char **model);

/* Hardware-aware rank selection, host only (paper section 6; first step of Algorithm 1).
 * For each layer, in the order given: among the entries of its measured latency table whose Tucker
 * MACs  P = H*W*C*R1 + Ho*Wo*K*K*R1*R2 + Ho*Wo*N*R2  (section 3; batch included) respect the FLOPs
 * budget, take those of minimal latency -- within the relative tolerance `tie_tol`, 0 for exact
 * ties only -- and among these the largest ranks (largest R1*R2, then R1+R2, then R1).  The layer
 * is decomposed only if that latency t1 < (1 - theta) * t2, t2 = dense_latency_us of its original
 * convolution (the paper uses theta = 0.15).
 * `budget` in [0,1) is the target MAC reduction ratio over all listed layers.  Layer l may keep at
 * most (1 - b_l) * F_l MACs, F_l = Ho*Wo*K*K*C*N, with
 *     b_l = max(0, (budget * sum_k F_k - MACs removed by layers before l) / sum_{k >= l} F_k),
 * so the share of a layer that stays dense passes to the layers after it.
 * R1, R2 and layout of `shape` are ignored.  Table entries of one layer must have distinct
 * (R1, R2), positive ranks and latencies.  out[l] receives the choice for layer l: decomposed = 1
 * with the ranks, their table latency and P, or decomposed = 0, R1 = R2 = 0, t2 and F_l.
 * Returns TDC_ERR_NULL or TDC_ERR_BAD_SHAPE on invalid arguments; never touches a device. */
typedef struct tdc_rank_entry {
    int32_t R1, R2;
    double latency_us;
} tdc_rank_entry;

typedef struct tdc_rank_layer {
    tdc_shape shape;
    const tdc_rank_entry *table;   /* host pointer, n_entries elements, caller-owned */
    int32_t n_entries;
    double dense_latency_us;
} tdc_rank_layer;

typedef struct tdc_rank_choice {
    int32_t decomposed;
    int32_t R1, R2;
    double latency_us;
    double macs;
} tdc_rank_choice;

int tdc_select_ranks(const tdc_rank_layer *layers, int n_layers, double budget, double theta,
                     double tie_tol, tdc_rank_choice *out);

/* Producer side of the format, HOST pointers, host only (paper section 4).
 * tdc_hosvd_tucker2: the projection of a dense kernel W[C][N][K][K] onto Tucker ranks (R1, R2) by
 * truncated HOSVD -- U_in[C][R1] = the R1 leading left singular vectors of the mode-1 matricization
 * (C x N*K*K), U_out[R2][N] = the transposed R2 leading left singular vectors of the mode-2
 * matricization (N x C*K*K), core[R1][R2][K][K] = W x_1 U_in^T x_2 U_out -- in the layouts
 * tdc_conv_tucker2 takes, so a pretrained layer can be decomposed and run.  Singular vectors are
 * determined up to sign; the sign that makes each vector's largest-magnitude component positive
 * is returned.  Requires 1 <= R1 <= C, 1 <= R2 <= N.  Arithmetic in fp64, results rounded to fp32.
 * tdc_admm_project: the two auxiliary updates of the ADMM training loop that need only that
 * projection:  K_hat <- proj(K + M)  (the tensor of Tucker ranks (R1, R2), in W's layout) and, in
 * place,  M <- M + K - K_hat.  The K update itself needs the training loss's gradient and is the
 * caller's; M is updated with the K_hat that is returned (rounded to fp32), so M_new = fp32(M + K - K_hat) holds for
 * the values the caller sees.  Cost is O(C^3 + N^3 + C*N*K*K*(C + N)) per call, meant to run offline.  Both return
 * TDC_ERR_NO_CONVERGENCE, and write nothing, if the Jacobi eigensolver does not reach its tolerance in 100 sweeps. */
int tdc_hosvd_tucker2(const float *W, int C, int N, int K, int R1, int R2,
                      float *U_in, float *core, float *U_out);
int tdc_admm_project(const float *K_weights, float *M, int C, int N, int K, int R1, int R2, float *K_hat);

/* Output size rule used everywhere: floor((in + 2*pad - K)/stride) + 1; returns 0 on bad input. */
int tdc_out_size(int in, int K, int stride, int pad);

#ifdef __cplusplus
}
#endif
#endif /* TDC_H */
