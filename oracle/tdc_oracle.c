/*
 * CPU oracle for a Tucker-2-format convolution layer  --  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, obviously-correct reference that the GPU library is
 * checked against.  It is not part of the product: only the tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it.  It shares no code,
 * header, table or helper with the HIP path.
 *
 * What it computes (paper section 3, "Basics of TKD-based Convolution"):
 *
 *   Eq. 1   K(c,n,r,s) = sum_{d1,d2} core(d1,d2,r,s) * U_in(c,d1) * U_out(d2,n)
 *   Eq. 2   Z1(h,w,d1)   = sum_c X(h,w,c) * U_in(c,d1)                (1x1 conv)
 *   Eq. 3   Z2(h',w',d2) = sum_{r,s,d1} Z1(h,w,d1) * core(d1,d2,r,s)  (core conv)
 *           with h = h'+r-1, w = w'+s-1 in the paper's 1-based, stride-1 form
 *   Eq. 4   Y(h',w',n)   = sum_{d2} Z2(h',w',d2) * U_out(d2,n)        (1x1 conv)
 *
 * and the plain definition the three stages are equivalent to (the paper's
 * equivalence claim after Eq. 4): a dense K x K cross-correlation of X with
 * the reconstructed kernel of Eq. 1.
 *
 * Readings taken where the paper is silent or inconsistent:
 *   - the core tensor is D1 x D2 x R x S, i.e. core[R1][R2][K][K] (the size
 *     printed below Eq. 1 is a misprint; the indexing in Eqs. 1 and 3 decides);
 *   - U_out is stored [R2][N], the view Eq. 4 uses; Eq. 1 reads the same
 *     matrix as U2(n,d2);
 *   - cross-correlation, no kernel flip (h = h'+r-1);
 *   - zero padding `pad` and stride apply to the core convolution's input Z1;
 *     stage 1 runs on all H x W pixels (the paper's cost formula counts
 *     H*W*C*D1 for it).  0-based: input row = i*stride + r - pad;
 *   - no bias, normalisation or activation anywhere: the layer is linear in X;
 *   - tensors are NCHW: x[B][C][H][W], z1[B][R1][H][W], z2[B][R2][Ho][Wo],
 *     y[B][N][Ho][Wo], Ho = floor((H + 2*pad - K)/stride) + 1.
 *
 * Arithmetic: inputs are fp32; every product, sum and intermediate is fp64.
 * Loops are written in the order of the equations; there is no blocking,
 * im2col, BLAS or vector intrinsic.  The only concession to run time is an
 * OpenMP "parallel for" over the outermost output-channel loop.
 *
 * Every routine returns the number of multiply-accumulates it visited
 * (padded taps included), so that tests can compare loop bounds with the
 * paper's complexity formula  H*W*C*D1 + H'*W'*R*S*D1*D2 + H'*W'*N*D2.
 */
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct orc_shape {
    int32_t batch, C, N, H, W; /* x is [batch][C][H][W]                     */
    int32_t R1, R2, K;         /* Tucker ranks D1, D2; square K x K filter  */
    int32_t stride, pad;       /* of the core convolution                   */
} orc_shape;

int orc_out_h(const orc_shape *s) { return (s->H + 2 * s->pad - s->K) / s->stride + 1; }
int orc_out_w(const orc_shape *s) { return (s->W + 2 * s->pad - s->K) / s->stride + 1; }

int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* Returns 0 when the shape describes a computable layer, else a negative code. */
int orc_check_shape(const orc_shape *s)
{
    if (!s) return -1;
    if (s->batch < 1 || s->C < 1 || s->N < 1 || s->H < 1 || s->W < 1) return -2;
    if (s->R1 < 1 || s->R2 < 1 || s->K < 1) return -2;
    if (s->stride < 1 || s->pad < 0) return -2;
    if (s->H + 2 * s->pad < s->K || s->W + 2 * s->pad < s->K) return -2;
    return 0;
}

/* Eq. 1: Wd[c][n][r][s] = sum_{d1} sum_{d2} core[d1][d2][r][s] * U_in[c][d1] * U_out[d2][n]. */
uint64_t orc_reconstruct(const orc_shape *sh, const float *U_in, const float *core,
                         const float *U_out, double *Wd)
{
    const int C = sh->C, N = sh->N, R1 = sh->R1, R2 = sh->R2, K = sh->K;
    uint64_t macs = 0;
#pragma omp parallel for reduction(+ : macs) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < K; ++r)
                for (int s = 0; s < K; ++s) {
                    double acc = 0.0;
                    for (int d1 = 0; d1 < R1; ++d1)
                        for (int d2 = 0; d2 < R2; ++d2) {
                            double cv = core[(((size_t)d1 * R2 + d2) * K + r) * K + s];
                            double u1 = U_in[(size_t)c * R1 + d1];
                            double u2 = U_out[(size_t)d2 * N + n];
                            acc += cv * u1 * u2;
                            ++macs;
                        }
                    Wd[(((size_t)c * N + n) * K + r) * K + s] = acc;
                }
    return macs;
}

/*
 * The definition: y[b][n][i][j] = sum_{c,r,s} xpad[b][c][i*stride+r-pad][j*stride+s-pad] * Wd[c][n][r][s],
 * xpad being x extended by zeros outside the image.
 */
uint64_t orc_conv_dense(const orc_shape *sh, const float *x, const double *Wd, double *y)
{
    const int B = sh->batch, C = sh->C, N = sh->N, H = sh->H, W = sh->W, K = sh->K;
    const int st = sh->stride, pad = sh->pad;
    const int Ho = orc_out_h(sh), Wo = orc_out_w(sh);
    uint64_t macs = 0;
    for (int b = 0; b < B; ++b) {
#pragma omp parallel for reduction(+ : macs) schedule(static)
        for (int n = 0; n < N; ++n)
            for (int i = 0; i < Ho; ++i)
                for (int j = 0; j < Wo; ++j) {
                    double acc = 0.0;
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < K; ++r)
                            for (int s = 0; s < K; ++s) {
                                const int h = i * st + r - pad;
                                const int w = j * st + s - pad;
                                ++macs;
                                if (h < 0 || h >= H || w < 0 || w >= W) continue; /* zero padding */
                                double xv = x[(((size_t)b * C + c) * H + h) * W + w];
                                acc += xv * Wd[(((size_t)c * N + n) * K + r) * K + s];
                            }
                    y[(((size_t)b * N + n) * Ho + i) * Wo + j] = acc;
                }
    }
    return macs;
}

/* Eq. 2: z1[b][d1][h][w] = sum_c x[b][c][h][w] * U_in[c][d1], on every input pixel. */
uint64_t orc_stage1(const orc_shape *sh, const float *x, const float *U_in, double *z1)
{
    const int B = sh->batch, C = sh->C, H = sh->H, W = sh->W, R1 = sh->R1;
    uint64_t macs = 0;
    for (int b = 0; b < B; ++b) {
#pragma omp parallel for reduction(+ : macs) schedule(static)
        for (int d1 = 0; d1 < R1; ++d1)
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w) {
                    double acc = 0.0;
                    for (int c = 0; c < C; ++c) {
                        double xv = x[(((size_t)b * C + c) * H + h) * W + w];
                        acc += xv * (double)U_in[(size_t)c * R1 + d1];
                        ++macs;
                    }
                    z1[(((size_t)b * R1 + d1) * H + h) * W + w] = acc;
                }
    }
    return macs;
}

/* Eq. 3 with stride and zero padding: z2[b][d2][i][j] = sum_{d1,r,s} z1pad[b][d1][i*st+r-pad][j*st+s-pad] * core[d1][d2][r][s]. */
uint64_t orc_core(const orc_shape *sh, const double *z1, const float *core, double *z2)
{
    const int B = sh->batch, H = sh->H, W = sh->W, R1 = sh->R1, R2 = sh->R2, K = sh->K;
    const int st = sh->stride, pad = sh->pad;
    const int Ho = orc_out_h(sh), Wo = orc_out_w(sh);
    uint64_t macs = 0;
    for (int b = 0; b < B; ++b) {
#pragma omp parallel for reduction(+ : macs) schedule(static)
        for (int d2 = 0; d2 < R2; ++d2)
            for (int i = 0; i < Ho; ++i)
                for (int j = 0; j < Wo; ++j) {
                    double acc = 0.0;
                    for (int r = 0; r < K; ++r)
                        for (int s = 0; s < K; ++s)
                            for (int d1 = 0; d1 < R1; ++d1) {
                                const int h = i * st + r - pad;
                                const int w = j * st + s - pad;
                                ++macs;
                                if (h < 0 || h >= H || w < 0 || w >= W) continue; /* zero padding */
                                double zv = z1[(((size_t)b * R1 + d1) * H + h) * W + w];
                                acc += zv * (double)core[(((size_t)d1 * R2 + d2) * K + r) * K + s];
                            }
                    z2[(((size_t)b * R2 + d2) * Ho + i) * Wo + j] = acc;
                }
    }
    return macs;
}

/* Eq. 4: y[b][n][i][j] = sum_{d2} z2[b][d2][i][j] * U_out[d2][n]. */
uint64_t orc_stage3(const orc_shape *sh, const double *z2, const float *U_out, double *y)
{
    const int B = sh->batch, N = sh->N, R2 = sh->R2;
    const int Ho = orc_out_h(sh), Wo = orc_out_w(sh);
    uint64_t macs = 0;
    for (int b = 0; b < B; ++b) {
#pragma omp parallel for reduction(+ : macs) schedule(static)
        for (int n = 0; n < N; ++n)
            for (int i = 0; i < Ho; ++i)
                for (int j = 0; j < Wo; ++j) {
                    double acc = 0.0;
                    for (int d2 = 0; d2 < R2; ++d2) {
                        double zv = z2[(((size_t)b * R2 + d2) * Ho + i) * Wo + j];
                        acc += zv * (double)U_out[(size_t)d2 * N + n];
                        ++macs;
                    }
                    y[(((size_t)b * N + n) * Ho + i) * Wo + j] = acc;
                }
    }
    return macs;
}

/*
 * The method, stage by stage (Eqs. 2, 3, 4 in that order).  z1 and z2 are
 * caller-provided scratch of B*R1*H*W and B*R2*Ho*Wo doubles.  macs3, when
 * not NULL, receives the three per-stage MAC counts.
 */
uint64_t orc_conv_factored(const orc_shape *sh, const float *x, const float *U_in, const float *core,
                           const float *U_out, double *z1, double *z2, double *y, uint64_t *macs3)
{
    uint64_t m1 = orc_stage1(sh, x, U_in, z1);
    uint64_t m2 = orc_core(sh, z1, core, z2);
    uint64_t m3 = orc_stage3(sh, z2, U_out, y);
    if (macs3) {
        macs3[0] = m1;
        macs3[1] = m2;
        macs3[2] = m3;
    }
    return m1 + m2 + m3;
}
