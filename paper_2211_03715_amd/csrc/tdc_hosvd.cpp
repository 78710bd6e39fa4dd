// Producer side of the Tucker-2 format, host only (paper section 4): the projection of a dense
// kernel onto Tucker ranks (R1, R2) by truncated HOSVD, and the two auxiliary updates of the ADMM
// training loop that need nothing but that projection (K-hat and M).  The K update needs the
// training loss's gradient and stays with the caller.
//
// proj(T), T in R^{C x N x K x K}: U1 = the R1 left singular vectors of the mode-1 matricization
// T_(1) (C x N*K*K) with the largest singular values, U2 likewise for T_(2) (N x C*K*K),
// core = T x_1 U1^T x_2 U2^T, K-hat = core x_1 U1 x_2 U2 (Eq. 1).  The left singular vectors of
// T_(m) are the eigenvectors of the Gram matrix T_(m) T_(m)^T, which is what is decomposed here:
// a cyclic Jacobi eigensolver in fp64 on a C x C (N x N) matrix, run once per layer offline --
// the same place in the workflow as the weight re-layout.  Everything is computed in fp64 and
// rounded to fp32 once.  Eigenvector signs are fixed (largest-magnitude component positive) so
// that results are reproducible.
#include <algorithm>
#include <cmath>
#include <cstddef>
#include <new>
#include <numeric>
#include <vector>

#include "tdc.h"

namespace {

// A (n x n, symmetric, row-major) -> eigenvalues in w, eigenvectors in the columns of V.  Returns false if the
// off-diagonal mass is still above the threshold after the last sweep (the basis is then not to be trusted).
bool jacobi_eigen(std::vector<double> &A, int n, std::vector<double> &w, std::vector<double> &V)
{
    V.assign((size_t)n * n, 0.0);
    for (int i = 0; i < n; ++i) V[(size_t)i * n + i] = 1.0;
    double diag2 = 0.0;
    for (int i = 0; i < n; ++i) diag2 += A[(size_t)i * n + i] * A[(size_t)i * n + i];
    bool converged = false;
    for (int sweep = 0; sweep <= 100; ++sweep) {
        double off2 = 0.0;
        for (int p = 0; p < n; ++p)
            for (int q = p + 1; q < n; ++q) off2 += A[(size_t)p * n + q] * A[(size_t)p * n + q];
        if (off2 <= 1e-30 * (diag2 + 2.0 * off2) || off2 == 0.0) {
            converged = true;
            break;
        }
        if (sweep == 100) break;           // the check above was the one after the last sweep
        for (int p = 0; p < n - 1; ++p)
            for (int q = p + 1; q < n; ++q) {
                const double apq = A[(size_t)p * n + q];
                if (apq == 0.0) continue;
                const double app = A[(size_t)p * n + p], aqq = A[(size_t)q * n + q];
                const double theta = (aqq - app) / (2.0 * apq);
                const double t = (theta >= 0.0 ? 1.0 : -1.0) / (std::fabs(theta) + std::sqrt(theta * theta + 1.0));
                const double c = 1.0 / std::sqrt(t * t + 1.0), s = t * c;
                for (int k = 0; k < n; ++k) {          // columns p, q
                    const double akp = A[(size_t)k * n + p], akq = A[(size_t)k * n + q];
                    A[(size_t)k * n + p] = c * akp - s * akq;
                    A[(size_t)k * n + q] = s * akp + c * akq;
                }
                for (int k = 0; k < n; ++k) {          // rows p, q
                    const double apk = A[(size_t)p * n + k], aqk = A[(size_t)q * n + k];
                    A[(size_t)p * n + k] = c * apk - s * aqk;
                    A[(size_t)q * n + k] = s * apk + c * aqk;
                }
                for (int k = 0; k < n; ++k) {
                    const double vkp = V[(size_t)k * n + p], vkq = V[(size_t)k * n + q];
                    V[(size_t)k * n + p] = c * vkp - s * vkq;
                    V[(size_t)k * n + q] = s * vkp + c * vkq;
                }
            }
        diag2 = 0.0;
        for (int i = 0; i < n; ++i) diag2 += A[(size_t)i * n + i] * A[(size_t)i * n + i];
    }
    w.resize(n);
    for (int i = 0; i < n; ++i) w[i] = A[(size_t)i * n + i];
    return converged;
}

// The `rank` leading left singular vectors of the n x m matrix T (rows = the mode being decomposed),
// as columns of U (n x rank, row-major).
bool leading_left_singular_vectors(const std::vector<double> &T, int n, size_t m, int rank, std::vector<double> &U)
{
    std::vector<double> G((size_t)n * n, 0.0), w, V;
    for (int i = 0; i < n; ++i)
        for (int j = i; j < n; ++j) {
            double s = 0.0;
            const double *a = &T[(size_t)i * m], *b = &T[(size_t)j * m];
            for (size_t k = 0; k < m; ++k) s += a[k] * b[k];
            G[(size_t)i * n + j] = G[(size_t)j * n + i] = s;
        }
    if (!jacobi_eigen(G, n, w, V)) return false;
    std::vector<int> order(n);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return w[a] > w[b]; });
    U.assign((size_t)n * rank, 0.0);
    for (int r = 0; r < rank; ++r) {
        const int col = order[r];
        int big = 0;
        for (int i = 1; i < n; ++i)
            if (std::fabs(V[(size_t)i * n + col]) > std::fabs(V[(size_t)big * n + col])) big = i;
        const double sign = V[(size_t)big * n + col] < 0.0 ? -1.0 : 1.0;
        for (int i = 0; i < n; ++i) U[(size_t)i * rank + r] = sign * V[(size_t)i * n + col];
    }
    return true;
}

// T (fp64, [C][N][KK]) -> U1 [C][R1], U2 [N][R2], core [R1][R2][KK]; false if an eigen-decomposition did not converge
bool hosvd(const std::vector<double> &T, int C, int N, int KK, int R1, int R2, std::vector<double> &U1,
           std::vector<double> &U2, std::vector<double> &core)
{
    if (!leading_left_singular_vectors(T, C, (size_t)N * KK, R1, U1)) return false;
    std::vector<double> T2((size_t)N * C * KK);                      // mode-2 matricization: [N][C][KK]
    for (int c = 0; c < C; ++c)
        for (int n = 0; n < N; ++n)
            for (int k = 0; k < KK; ++k) T2[((size_t)n * C + c) * KK + k] = T[((size_t)c * N + n) * KK + k];
    if (!leading_left_singular_vectors(T2, N, (size_t)C * KK, R2, U2)) return false;
    std::vector<double> A((size_t)R1 * N * KK, 0.0);                 // T x_1 U1^T : [R1][N][KK]
    for (int c = 0; c < C; ++c)
        for (int d1 = 0; d1 < R1; ++d1) {
            const double u = U1[(size_t)c * R1 + d1];
            const double *src = &T[(size_t)c * N * KK];
            double *dst = &A[(size_t)d1 * N * KK];
            for (size_t k = 0; k < (size_t)N * KK; ++k) dst[k] += u * src[k];
        }
    core.assign((size_t)R1 * R2 * KK, 0.0);                          // x_2 U2^T : [R1][R2][KK]
    for (int d1 = 0; d1 < R1; ++d1)
        for (int n = 0; n < N; ++n)
            for (int d2 = 0; d2 < R2; ++d2) {
                const double u = U2[(size_t)n * R2 + d2];
                for (int k = 0; k < KK; ++k) core[((size_t)d1 * R2 + d2) * KK + k] += u * A[((size_t)d1 * N + n) * KK + k];
            }
    return true;
}

bool bad_dims(int C, int N, int K, int R1, int R2)
{
    return C < 1 || N < 1 || K < 1 || R1 < 1 || R2 < 1 || R1 > C || R2 > N || (double)C * N * K * K >= 2147483647.0;
}

}  // namespace

extern "C" int tdc_hosvd_tucker2(const float *W, int C, int N, int K, int R1, int R2, float *U_in, float *core, float *U_out)
{
    if (!W || !U_in || !core || !U_out) return TDC_ERR_NULL;
    if (bad_dims(C, N, K, R1, R2)) return TDC_ERR_BAD_SHAPE;
    const int KK = K * K;
    try {
        std::vector<double> T((size_t)C * N * KK), U1, U2, G;
        for (size_t i = 0; i < T.size(); ++i) T[i] = W[i];
        if (!hosvd(T, C, N, KK, R1, R2, U1, U2, G)) return TDC_ERR_NO_CONVERGENCE;
        for (size_t i = 0; i < U1.size(); ++i) U_in[i] = (float)U1[i];
        for (size_t i = 0; i < G.size(); ++i) core[i] = (float)G[i];
        for (int n = 0; n < N; ++n)
            for (int d2 = 0; d2 < R2; ++d2) U_out[(size_t)d2 * N + n] = (float)U2[(size_t)n * R2 + d2];
    } catch (const std::bad_alloc &) {
        return TDC_ERR_ALLOC;
    }
    return TDC_OK;
}

extern "C" int tdc_admm_project(const float *Kw, float *M, int C, int N, int K, int R1, int R2, float *K_hat)
{
    if (!Kw || !M || !K_hat) return TDC_ERR_NULL;
    if (bad_dims(C, N, K, R1, R2)) return TDC_ERR_BAD_SHAPE;
    const int KK = K * K;
    try {
        std::vector<double> T((size_t)C * N * KK), U1, U2, G;
        for (size_t i = 0; i < T.size(); ++i) T[i] = (double)Kw[i] + (double)M[i];
        if (!hosvd(T, C, N, KK, R1, R2, U1, U2, G)) return TDC_ERR_NO_CONVERGENCE;   // K_hat and M untouched
        // K-hat = core x_1 U1 x_2 U2, then M <- M + K - K-hat with the K-hat the caller receives (rounded to fp32)
        std::vector<double> A((size_t)R1 * N * KK, 0.0);             // core x_2 U2 : [R1][N][KK]
        for (int d1 = 0; d1 < R1; ++d1)
            for (int d2 = 0; d2 < R2; ++d2)
                for (int n = 0; n < N; ++n) {
                    const double u = U2[(size_t)n * R2 + d2];
                    for (int k = 0; k < KK; ++k) A[((size_t)d1 * N + n) * KK + k] += u * G[((size_t)d1 * R2 + d2) * KK + k];
                }
        std::vector<double> row((size_t)N * KK);
        for (int c = 0; c < C; ++c) {
            std::fill(row.begin(), row.end(), 0.0);
            for (int d1 = 0; d1 < R1; ++d1) {
                const double u = U1[(size_t)c * R1 + d1];
                const double *src = &A[(size_t)d1 * N * KK];
                for (size_t k = 0; k < row.size(); ++k) row[k] += u * src[k];
            }
            for (size_t k = 0; k < row.size(); ++k) {
                const size_t i = (size_t)c * N * KK + k;
                K_hat[i] = (float)row[k];
                M[i] = (float)((double)M[i] + (double)Kw[i] - (double)K_hat[i]);
            }
        }
    } catch (const std::bad_alloc &) {
        return TDC_ERR_ALLOC;
    }
    return TDC_OK;
}
