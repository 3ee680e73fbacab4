// Internal declarations of the offline quantizer's translation units (not installed).
// Everything here computes in fp64 on device-resident arrays; the launchers enqueue on the given
// stream and never synchronize or allocate.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "bwla_quantizer.h"

// ---------------------------------------------------------------- fp64 GEMM (quantizer_gemm.hip)
// C[b] = alpha * A[b] * B[b] + beta * C0[b], fp64 MFMA 16x16x4, 64 x 64 tiles.
// Operands are addressed through strides so that views of the quantizer's n x m arrays (rows
// reshaped to n1 x n2, transposes, sums over the rows of all reshaped matrices) need no copies:
//   A(i, k) = A[b * bsA + i * rsA + (k / kdivA) * khA + (k % kdivA) * klA]
//   B(k, j) = B[b * bsB + j * csB + (k / kdivB) * khB + (k % kdivB) * klB]
//   C(i, j) = C[b * bsC + i * rsC + j]            (C0 is addressed like C)
// kdiv = 0 stands for "no split of the contraction index" (k / kdiv = 0, k % kdiv = k).
// ksplit > 1 cuts the contraction into ksplit ranges whose partial products go to `partials`
// (ksplit x batch x M x N, dense) and are added in range order by a second launch, which also
// applies alpha, beta and C0: deterministic whatever the launch order.
// `skip` (device, may be NULL): when *skip != 0 the launches return without touching C.
struct QGemm {
    const double* A; const double* B; double* C; const double* C0;
    int M, N, K, batch;
    long rsA, khA, klA, bsA; int kdivA;
    long csB, khB, klB, bsB; int kdivB;
    long rsC, bsC;
    double alpha, beta;
    int ksplit; double* partials;
    const int* skip;
};
inline QGemm qgemm_plain(const double* A, const double* B, double* C, int M, int N, int K) {
    QGemm g{};
    g.A = A; g.B = B; g.C = C; g.C0 = nullptr; g.M = M; g.N = N; g.K = K; g.batch = 1;
    g.rsA = K; g.klA = 1; g.csB = 1; g.klB = N; g.rsC = N; g.alpha = 1.0; g.beta = 0.0; g.ksplit = 1;
    return g;
}
hipError_t bwla_q_launch_gemm(const QGemm& g, hipStream_t st);
inline size_t bwla_q_gemm_partial_bytes(int M, int N, int batch, int ksplit) {
    return ksplit > 1 ? (size_t)ksplit * batch * M * N * sizeof(double) : 0;
}

// ---------------------------------------------------------------- row kernels (quantizer_rows.hip)
hipError_t bwla_q_launch_convert_f32_f64(const float* src, double* dst, size_t count, hipStream_t st);
hipError_t bwla_q_launch_convert_f64_f32(const double* src, float* dst, size_t count, hipStream_t st);
// X = Y - row means (X may be NULL: only the means), ybar = the means (may be NULL)
hipError_t bwla_q_launch_center(const double* Y, double* X, double* ybar, int n, int m, hipStream_t st);
hipError_t bwla_q_launch_init_theta(const double* X, int n, int m, double s2_min, double* c, double* s2, hipStream_t st);
hipError_t bwla_q_launch_em(const double* X, int n, int m, double s2_min, double* c, double* s2, hipStream_t st);
// out[0] = L_GMM; row_part: n doubles of scratch
hipError_t bwla_q_launch_nll(const double* X, int n, int m, const double* c, const double* s2, double* row_part,
                             double* out, hipStream_t st);
// T = lambda_i * (H m_i + ybar_i 1), m_ij = c_i tanh(c_i x_ij / s_i^2), x = y - ybar
hipError_t bwla_q_launch_targets(const double* Y, const double* ybar, const double* c, const double* s2, int n, int m,
                                 double* T, hipStream_t st);
// fac[0] = mu > 0 ? 1 / (n m mu) : min_i s2_i   (the factor that turns (x - m) lambda into -(grad_X) / mu)
hipError_t bwla_q_launch_prox_factor(const double* s2, int n, int m, double mu, double* fac, hipStream_t st);
// GX = fac * H[(x - m) lambda]
hipError_t bwla_q_launch_gradx(const double* X, const double* c, const double* s2, const double* fac, int n, int m,
                               double* GX, hipStream_t st);
// Q[i] = uniform in [-1, 1) from a counter-based hash of (seed, i)
hipError_t bwla_q_launch_fill_hash(double* Q, size_t count, uint32_t seed, hipStream_t st);
hipError_t bwla_q_launch_fill_identity(double* R, int n, hipStream_t st);
// X = C / ||C||_F (count values, one workgroup; a zero matrix stays zero)
hipError_t bwla_q_launch_scale_inv_frob(const double* C, int count, double* X, hipStream_t st);
// out[0] = 1 / sqrt(max_j sum_i |G_ij|) for a Gram matrix G = X^T X (nn x nn): a bound on 1 / sigma_max(X)
// (0 for a zero matrix); one workgroup
hipError_t bwla_q_launch_gram_inv_norm(const double* G, int nn, double* out, hipStream_t st);
// X[e] *= s[0]
hipError_t bwla_q_launch_scale_by(double* X, size_t count, const double* s, hipStream_t st);
// *done = 1 once max |G - I| <= tol (G nn x nn); never cleared
hipError_t bwla_q_launch_near_identity(const double* G, int nn, double tol, int* done, hipStream_t st);
hipError_t bwla_q_launch_set_int(int* p, int v, hipStream_t st);
hipError_t bwla_q_launch_fill_value(double* p, size_t count, double v, hipStream_t st);
// dst[e] = src[e]^pw (0 where src <= 0)
hipError_t bwla_q_launch_pow_vec(const double* src, double pw, int count, double* dst, hipStream_t st);
// dst[i][j] = src[i][j] * pow(lam[j], pw) (fp32 out, n x k; lam <= 0 gives 0)
hipError_t bwla_q_launch_scale_cols_f32(const double* src, const double* lam, double pw, int n, int k, float* dst,
                                        hipStream_t st);
// row-wise binarization statistics of Algorithm 2's last step: mu_i = mean_j y_ij, alpha_i = mean_j |y_ij - mu_i|
hipError_t bwla_q_launch_row_stats(const double* Y, int n, int m, double* mean, double* absdev, hipStream_t st);

// ---------------------------------------------------------------- one-sided Jacobi (quantizer_jacobi.hip)
// Singular value decomposition G = U S V^T of a square n x n matrix (n <= 256) by Hestenes'
// one-sided Jacobi rotations in one workgroup.  Outputs, ordered by descending singular value:
//   sig[j]        singular values
//   Ws[j][:]      column j of G V = s_j u_j            (n x n, row j = that column)
//   Vs[j][:]      s_j^pw * v_j                          (n x n, row j = that vector; s_j = 0 gives 0)
// `work` holds 2 n^2 doubles.  conv (may be NULL): {int done; } convergence bookkeeping of the subspace
// iteration -- when prev_sig is given, done is set once the leading `lead` singular values moved by
// at most tol relative to the previous call, and prev_sig is replaced.  The launch returns
// immediately when *skip != 0.
// sym: G is symmetric positive semidefinite (a Gram matrix): the rotations are not accumulated, v_j is
// the normalized column j of G V (equal to u_j there), and matrices up to 136 wide stay in LDS.
struct QJacobi {
    const double* G; int n; double pw;
    double* sig; double* Ws; double* Vs; double* work;
    double* prev_sig; int lead; double tol; int* done; const int* skip;
    bool sym;
};
hipError_t bwla_q_launch_jacobi(const QJacobi& j, hipStream_t st);
constexpr int BWLA_Q_JACOBI_LDS = 96;        // largest matrix whose two work arrays fit LDS
constexpr int BWLA_Q_JACOBI_SYM_LDS = 136;   // ... whose one array does (sym)
