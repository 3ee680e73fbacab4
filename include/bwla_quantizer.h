/*
 * bwla_quantizer.h -- C ABI of the offline quantizer of BWLA on MI355X (gfx950): the procedure that
 * produces what bwla_pack_weights consumes (paper App. A.1, Algorithm 2 "Quantization Framework of
 * BWLA"; Sec. 3.1 for the Orthogonal-Kronecker Transformation and its EM / MM updates, App. A.2.2
 * for their derivation; Sec. 3.2 and App. A.2.3 for the Proximal SVD Projection).
 *
 * For a weight matrix W (n rows = output channels, m = n1 n2 columns) the procedure alternates
 *   X = (W - M) (R1 (x) R2) H,  H = I - 1 1^T / m              OKT-centered rows
 *   EM      row-wise symmetric two-component Gaussian mixture: r_ij, then c_i, s_i^2
 *   PSP     M <- rank-k truncation of M - (1 / mu) dL_GMM/dM    (proximal step, truncated SVD)
 *   MM      R1, then R2 <- the orthogonal Procrustes solutions for the targets (2 r_ij - 1) c_i
 *           with weights 1 / s_i^2
 * and ends with W_rot = (W - M)(R1 (x) R2), which bwla_pack_weights_centered binarizes row by row.
 *
 * Everything is computed in fp64 on the GPU, with the dense contractions on fp64 MFMA.  Conventions
 * as in bwla.h: device pointers owned by the caller, at least 16-byte aligned, dense row-major;
 * calls enqueue on `stream` and do not synchronize, allocate nothing, and validate their arguments
 * on the host before anything is enqueued (status codes of bwla.h).  The Kronecker convention is
 * the forward path's: a row times R1 (x) R2 is R1^T V R2 on the row reshaped row-major to n1 x n2.
 * Limits (BWLA_ERR_UNSUPPORTED): n1, n2 <= 256; k <= 128; n <= 65535; m <= 65536.
 *
 * Readings of the paper taken here (the same as the test oracle's, each derived in its header):
 * the MM targets of a row are the centered targets plus the row's current mean (this makes every
 * Procrustes update an exact majorize-minimize step of the centered likelihood); s_i^2 is updated
 * with the new c_i; the proximal point is M - (1 / mu) dL/dM with dL/dM = -(G_X H) R^T; the default
 * mu is 1 / (n m min_i s_i^2), for which the quadratic model majorizes L_GMM globally.
 */
#ifndef BWLA_QUANTIZER_H
#define BWLA_QUANTIZER_H

#include "bwla.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Bytes of scratch that every call below accepts for a problem of this size (five n x m fp64
 * arrays, the subspace-iteration blocks, Jacobi work space, split-contraction partial sums): the d_ws
 * of a call must hold at least as many, except where a call states a smaller need.  n1 = n2 = 1 with
 * m > 1 sizes the scratch of the calls that take no factors (bwla_q_truncate_rank).  Host only. */
BWLA_API bwla_status_t bwla_quantizer_workspace_size(int64_t n, int64_t m, int32_t n1, int32_t n2, int32_t k,
                                                     size_t* bytes);

/*
 * X = ((W - A Bt^T)(R1 (x) R2)) H  (Sec. 3.2, the transform T_R applied to the corrected weight).
 *   d_W   n x m;  d_A  n x k and d_Bt  m x k, the low-rank term M = A Bt^T (both NULL iff k == 0)
 *   d_R1  n1 x n1, d_R2  n2 x n2;  d_X out, n x m;  d_ybar out (may be NULL): the n row means taken out
 */
BWLA_API bwla_status_t bwla_q_okt_rows(const double* d_W, const double* d_A, const double* d_Bt, int32_t k,
                                       const double* d_R1, const double* d_R2, int64_t n, int64_t m, int32_t n1,
                                       int32_t n2, double* d_X, double* d_ybar, void* d_ws, size_t ws_bytes,
                                       void* stream);

/* Algorithm 2, "initialize c_i, s_i^2 from W": c_i = mean_j |x_ij|, s_i^2 = mean_j (|x_ij| - c_i)^2,
 * floored at s2_min.  d_c, d_s2 out, n each. */
BWLA_API bwla_status_t bwla_q_init_theta(const double* d_X, int64_t n, int64_t m, double s2_min, double* d_c,
                                         double* d_s2, void* stream);

/* One EM update of the row mixtures (App. A.2.2): responsibilities at (c, s^2), then
 * c_i = mean_j (2 r_ij - 1) x_ij and, with that c_i, s_i^2 = mean_j [r (x - c)^2 + (1 - r)(x + c)^2],
 * floored at s2_min.  d_c, d_s2 in and out. */
BWLA_API bwla_status_t bwla_q_em_step(const double* d_X, int64_t n, int64_t m, double s2_min, double* d_c,
                                      double* d_s2, void* stream);

/* L_GMM (App. A.2.2): -1 / (n m) sum_ij log[ 1/2 phi(x_ij; c_i, s_i^2) + 1/2 phi(x_ij; -c_i, s_i^2) ]
 * to d_out[0].  d_ws: n fp64 values are enough. */
BWLA_API bwla_status_t bwla_q_gmm_nll(const double* d_X, int64_t n, int64_t m, const double* d_c,
                                      const double* d_s2, double* d_out, void* d_ws, size_t ws_bytes,
                                      void* stream);

/*
 * One Procrustes update of the MM step (App. A.2.2, "Alternating Procrustes Updates"), targets and
 * weights taken at the given factors: which = 1 gives the minimizer over R1 of
 * sum_i lambda_i || R1^T V_i R2 - T_i ||_F^2 (polar factor of C1 = sum_i lambda_i V_i R2 T_i^T),
 * which = 2 the minimizer over R2 (C2 = sum_i lambda_i V_i^T R1 T_i); V_i is row i of d_Wres = W - M
 * reshaped, T_i its target.  d_Rnew out, n1 x n1 or n2 x n2.  The polar factor comes from a one-sided
 * Jacobi SVD for factors up to 64 and from the Newton-Schulz iteration X <- X (3 I - X^T X) / 2 on
 * C / ||C||_F above (the same matrix, from small GEMMs instead of a single workgroup); a singular C
 * has no unique one and gives an undefined (finite) result.
 */
BWLA_API bwla_status_t bwla_q_procrustes(int32_t which, const double* d_Wres, const double* d_R1,
                                         const double* d_R2, const double* d_c, const double* d_s2, int64_t n,
                                         int64_t m, int32_t n1, int32_t n2, double* d_Rnew, void* d_ws,
                                         size_t ws_bytes, void* stream);

/*
 * SVD of a square matrix, nn <= 256, by one-sided Jacobi rotations: d_sig (nn, descending),
 * d_Ut (row j = left singular vector j times sigma_j), d_Vt (row j = right singular vector j).
 * Any of the three outputs may be NULL.  d_ws: 2 nn^2 fp64 values are enough.
 */
BWLA_API bwla_status_t bwla_q_svd_square(const double* d_G, int32_t nn, double* d_sig, double* d_Ut, double* d_Vt,
                                         void* d_ws, size_t ws_bytes, void* stream);

/*
 * Best rank-k approximation of Y (n x m) in the Frobenius norm (Sec. 3.2: the projection onto the
 * rank-k matrices is the truncated SVD), returned in factors: Y_k = A Bt^T with A = Y V_k (n x k,
 * column j = sigma_j u_j) and Bt = V_k (m x k, orthonormal columns); d_sig (may be NULL) gets the k
 * singular values.  Computed by block subspace iteration on Y^T Y with a block of
 * min(n, m, max(2 k, k + 16)) vectors from a fixed pseudo-random start, re-orthonormalized every
 * iteration through the eigendecomposition of its Gram matrix, and a final Rayleigh-Ritz step.  It
 * stops after `iters` iterations, or earlier once the k leading Ritz values have moved by at most
 * `tol` (relative) in one iteration: the remaining launches then return at once.  (Blocks of more than
 * 136 vectors, i.e. k > 68, are orthonormalized by the Newton-Schulz iteration instead, have no Ritz
 * values along the way and always run all `iters` iterations.)  The captured
 * energy converges like (sigma_{p+1} / sigma_k)^(4 iterations); a spectrum without a gap behind
 * sigma_k needs many iterations for the singular vectors themselves.
 * d_ws: bwla_quantizer_workspace_size(n, m, 1, 1, k) bytes.
 */
BWLA_API bwla_status_t bwla_q_truncate_rank(const double* d_Y, int64_t n, int64_t m, int32_t k, int32_t iters,
                                            double tol, double* d_A, double* d_Bt, double* d_sig, void* d_ws,
                                            size_t ws_bytes, void* stream);

/*
 * The PSP update (Sec. 3.2; App. A.2.3): M <- rank-k truncation of M - (1 / mu) dL_GMM(W - M)/dM at the
 * given factors and mixture parameters; d_A (n x k), d_Bt (m x k) hold M = A Bt^T on entry (the zero
 * matrix when both are zero-filled) and the new factors on return.  mu <= 0 selects the default
 * 1 / (n m min_i s_i^2).  iters, tol as in bwla_q_truncate_rank.
 */
BWLA_API bwla_status_t bwla_q_psp_step(const double* d_W, double* d_A, double* d_Bt, int32_t k, const double* d_R1,
                                       const double* d_R2, const double* d_c, const double* d_s2, int64_t n,
                                       int64_t m, int32_t n1, int32_t n2, double mu, int32_t iters, double tol,
                                       void* d_ws, size_t ws_bytes, void* stream);

/*
 * Algorithm 2 on one weight matrix: t_outer rounds of { EM, PSP (when k > 0), Procrustes update of R1,
 * then of R2 }, starting from M = 0 and the given factors.
 *   d_W      n x m fp32
 *   d_R1, d_R2  fp32 factors, in and out: the start (init_identity = 0) or ignored on entry and started
 *            at the identity (init_identity = 1); on return the learned factors
 *   d_W_rot  out, n x m fp32: (W - M)(R1 (x) R2), the matrix bwla_pack_weights[_centered] binarizes
 *   d_U      out, m x k fp32 and d_V out, n x k fp32: the balanced factors of M = V U^T
 *            (V = U_k S_k^(1/2), U = V_k S_k^(1/2): App. A.2.3), the arguments of the same name of
 *            bwla_pack_weights; NULL iff k == 0
 *   d_c, d_s2   out, n fp64 each: the mixture parameters (may be NULL)
 *   d_hist   out (may be NULL): 1 + 3 t_outer fp64 values of L_GMM -- at the start, then after the EM,
 *            the PSP and the MM step of every round (the PSP entry repeats the EM one when k == 0)
 *   mu, svd_iters, svd_tol  as in bwla_q_psp_step; s2_min the floor of s_i^2
 */
BWLA_API bwla_status_t bwla_quantize_layer(const float* d_W, int64_t n, int64_t m, int32_t n1, int32_t n2, int32_t k,
                                           int32_t t_outer, double mu, double s2_min, int32_t svd_iters,
                                           double svd_tol, int32_t init_identity, float* d_R1, float* d_R2,
                                           float* d_W_rot, float* d_U, float* d_V, double* d_c, double* d_s2,
                                           double* d_hist, void* d_ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BWLA_QUANTIZER_H */
