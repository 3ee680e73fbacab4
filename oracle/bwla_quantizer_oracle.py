"""CPU oracle of BWLA's offline quantizer (paper App. A.1, Algorithm 2; Sec. 3.1-3.2; App. A.2.2,
"Details of the Orthogonal-Kronecker Transformation"; App. A.2.3, "Detailed Derivations of the
Proximal SVD Projection").

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT: plain NumPy in fp64, the algorithm's steps in the
paper's order and notation, no blocking or fusion.  Only the tests may import it.

What is computed, for a weight matrix W (n rows = output channels, m = n1 n2 columns):

    X = (W - M) R H,  R = R1 (x) R2,  H = I - 1 1^T / m        the OKT-centered rows   (Sec. 3.2, T_R)
    L_GMM = -1/(n m) sum_ij log[ 1/2 phi(x_ij; c_i, s_i^2) + 1/2 phi(x_ij; -c_i, s_i^2) ]
    E step   r_ij = phi(x; c, s^2) / (phi(x; c, s^2) + phi(x; -c, s^2))
    M step   c_i = mean_j (2 r_ij - 1) x_ij,  s_i^2 = mean_j [r (x - c)^2 + (1 - r)(x + c)^2] >= s_min^2
    MM       targets m_ij = (2 r_ij - 1) c_i, weights lambda_i = 1 / s_i^2,
             surrogate 1/(n m) sum_i lambda_i || rot(V_i) - M_i ||_F^2, minimized over one factor at a
             time by an orthogonal Procrustes problem (SVD of an n1 x n1 or n2 x n2 matrix)
    PSP      gradient of L_GMM with respect to M, proximal point Y = M - grad / mu, M <- best rank-k
             approximation of Y (truncated SVD)
    final    row-wise binarization of (W - M) R with the row mean as shift

Readings taken where the paper is ambiguous or inconsistent (each is listed in the design notes):
  * Kronecker convention: the same as the forward path's, x (R1 (x) R2) = vec(R1^T V R2) on the
    row-major n1 x n2 reshape V.  The Procrustes matrices follow from that convention by the
    paper's own derivation: C1 = sum_i lambda_i V_i R2 M_i^T, C2 = sum_i lambda_i V_i^T R1 M_i
    (the paper prints them for its R2^T V R1 form).
  * V_i is the reshaped row of W - M (not of the already rotated matrix): the surrogate of
    App. A.2.2 is a function of the whole factors.
  * Centering inside the MM step.  The paper's Procrustes formulas are written for the rotated rows
    y_i = rot(v_i) while the likelihood sees x_i = H y_i.  Exactly, sum_j (x_ij - m_ij)^2 =
    ||y_i - H m_i||^2 - m mean(y_i)^2 + const, and the concave last term is majorized by its tangent
    at the current point, which turns the whole into ||y_i - (H m_i + mean(y_i^0) 1)||^2 + const:
    the Procrustes targets are the centered targets plus the row's current mean (mm_row_targets).
    With them every update is an exact MM step and L_GMM cannot increase; with the bare m_ij it can
    (and does, on Gaussian rows).
  * The M step uses the new c_i inside s_i^2 (the joint maximizer of the expected complete-data
    log-likelihood; Algorithm 2 lists the two updates in that order).
  * Gradient sign: with X = T_R(W - M), dL/dM = -T_R^*(dL/dX) = -(G_X H^T R^T).  The proximal point
    is M - (1/mu) dL/dM; taking the paper's G = +T_R^*(G_X) literally would ascend.
  * mu: any mu >= 1 / (n m min_i s_i^2) makes the quadratic model a global majorizer (the second
    derivative of -log p in x is at most 1 / s_i^2, and x -> x R H does not expand); that bound is
    the default.
  * Final binarization: per output channel = row (Sec. 3 "Discussion", Eq. 1-2), although Algorithm 2
    indexes it by column: the row mean is the shift, the row mean of |x - shift| the scale.

Pins (tests/test_quantizer_oracle.py): responsibilities against scipy's normal density; the M
step against a brute-force grid of the expected log-likelihood; EM never increases L_GMM; the
quadratic surrogate majorizes -log p and touches it at the current point; the Kronecker form of the
surrogate against a dense Kronecker product; each Procrustes update against
scipy.linalg.orthogonal_procrustes and against random orthogonal matrices, and the surrogate never
increases; the PSP gradient against central finite differences; the truncated SVD against random
rank-k candidates; L(W - M) never increases under the PSP step with the default mu; the whole loop's
history.  **Parity unpinned:** that the procedure finds a *good* quantizer (lower perplexity) --
the paper shows that only on pretrained models.
"""
from __future__ import annotations

import numpy as np

from oracle import bwla_oracle as fwd

S2_MIN = 1e-8


# --------------------------------------------------------------------------- OKT-centered rows
def center_rows(Y: np.ndarray) -> np.ndarray:
    """Y H with H = I - 1 1^T / m (Sec. 3.1, "Transformation Objectives")."""
    Y = np.asarray(Y, dtype=np.float64)
    return Y - Y.mean(axis=1, keepdims=True)


def okt_rows(W, M, R1, R2) -> np.ndarray:
    """X = (W - M) R H (Sec. 3.2, T_R applied to the corrected weight)."""
    return center_rows(fwd.kron_rotate(np.asarray(W, np.float64) - np.asarray(M, np.float64), R1, R2))


# --------------------------------------------------------------------------- symmetric two-component mixture
def gmm_nll(X, c, s2) -> float:
    """L_GMM (App. A.2.2, normalized negative log-likelihood), evaluated in log space."""
    X = np.asarray(X, np.float64)
    c = np.asarray(c, np.float64)[:, None]
    s2 = np.asarray(s2, np.float64)[:, None]
    lp = -0.5 * np.log(2.0 * np.pi * s2) - (X - c) ** 2 / (2.0 * s2)
    lm = -0.5 * np.log(2.0 * np.pi * s2) - (X + c) ** 2 / (2.0 * s2)
    return float(-np.mean(np.logaddexp(lp, lm) + np.log(0.5)))


def responsibilities(X, c, s2) -> np.ndarray:
    """r^+_ij (App. A.2.2, E step): the ratio of the two densities is exp(2 c x / s^2)."""
    X = np.asarray(X, np.float64)
    t = 2.0 * np.asarray(c, np.float64)[:, None] * X / np.asarray(s2, np.float64)[:, None]
    return 0.5 * (1.0 + np.tanh(0.5 * t))          # = 1 / (1 + exp(-t)), without overflow


def m_step(X, r, s2_min: float = S2_MIN):
    """Closed-form M step (App. A.2.2): c_i, then s_i^2 with the new c_i, floored at s2_min."""
    X = np.asarray(X, np.float64)
    c = np.mean((2.0 * r - 1.0) * X, axis=1)
    cc = c[:, None]
    s2 = np.mean(r * (X - cc) ** 2 + (1.0 - r) * (X + cc) ** 2, axis=1)
    return c, np.maximum(s2, s2_min)


def em_step(X, c, s2, s2_min: float = S2_MIN):
    r = responsibilities(X, c, s2)
    return m_step(X, r, s2_min)


def init_theta(X, s2_min: float = S2_MIN):
    """Empirical start (Algorithm 2, "initialize c_i, s_i^2 from W"): the two half-normal modes of
    a centered row, c = mean |x|, s^2 = mean (|x| - c)^2."""
    A = np.abs(np.asarray(X, np.float64))
    c = A.mean(axis=1)
    s2 = np.maximum(((A - c[:, None]) ** 2).mean(axis=1), s2_min)
    return c, s2


# --------------------------------------------------------------------------- MM surrogate and Procrustes steps
def mm_targets(X, c, s2):
    """m_ij = (2 r_ij - 1) c_i and lambda_i = 1 / s_i^2 (App. A.2.2, "MM Surrogate")."""
    r = responsibilities(X, c, s2)
    return (2.0 * r - 1.0) * np.asarray(c, np.float64)[:, None], 1.0 / np.asarray(s2, np.float64)


def mm_row_targets(Wres, R1, R2, c, s2):
    """Targets for the uncentered rotated rows y_i and the weights lambda_i: H m_i + mean(y_i) 1 at
    the current factors (see the readings in the header).  The surrogate built from them touches
    L_GMM (up to the factor 1/2 and a constant) at the current factors and majorizes it elsewhere."""
    Y = fwd.kron_rotate(Wres, R1, R2)
    ybar = Y.mean(axis=1, keepdims=True)
    m_ij, lam = mm_targets(Y - ybar, c, s2)
    return center_rows(m_ij) + ybar, lam


def surrogate(Wres, R1, R2, targets, lam) -> float:
    """1/(n m) sum_i lambda_i || R1^T V_i R2 - M_i ||_F^2 on the uncentered rotated rows."""
    Y = fwd.kron_rotate(Wres, R1, R2)
    n, m = Y.shape
    return float(np.sum(lam[:, None] * (Y - targets) ** 2) / (n * m))


def procrustes_r1(Wres, R2, targets, lam, n1: int, n2: int) -> np.ndarray:
    """argmin over orthogonal R1 of the surrogate with R2 fixed: C1 = sum_i lambda_i V_i R2 M_i^T,
    R1 = U V^T from the SVD of C1 (App. A.2.2, "Alternating Procrustes Updates", in this build's
    Kronecker convention)."""
    V = np.asarray(Wres, np.float64).reshape(-1, n1, n2)
    Mi = np.asarray(targets, np.float64).reshape(-1, n1, n2)
    C1 = np.einsum("i,iab,bd,icd->ac", lam, V, np.asarray(R2, np.float64), Mi)
    U, _, Vt = np.linalg.svd(C1)
    return U @ Vt


def procrustes_r2(Wres, R1, targets, lam, n1: int, n2: int) -> np.ndarray:
    """The same with R1 fixed: C2 = sum_i lambda_i V_i^T R1 M_i, R2 = U V^T."""
    V = np.asarray(Wres, np.float64).reshape(-1, n1, n2)
    Mi = np.asarray(targets, np.float64).reshape(-1, n1, n2)
    C2 = np.einsum("i,iab,ac,icd->bd", lam, V, np.asarray(R1, np.float64), Mi)
    U, _, Vt = np.linalg.svd(C2)
    return U @ Vt


# --------------------------------------------------------------------------- proximal SVD projection
def grad_x(X, c, s2) -> np.ndarray:
    """dL_GMM / dx_ij = (x_ij - m_ij) / (n m s_i^2) (App. A.2.2, gradient with respect to the entries)."""
    m_ij, lam = mm_targets(X, c, s2)
    n, m = X.shape
    return (np.asarray(X, np.float64) - m_ij) * lam[:, None] / (n * m)


def grad_m(W, M, R1, R2, c, s2) -> np.ndarray:
    """dL(W - M) / dM = -(G_X H^T) R^T (App. A.2.3, "Adjoint of the OKT Transform", with the sign of
    delta X = -T_R(delta M) kept)."""
    X = okt_rows(W, M, R1, R2)
    GX = center_rows(grad_x(X, c, s2))                                  # G_X H^T (H is symmetric)
    # rows times R^T = (R1 (x) R2)^T = R1^T (x) R2^T
    return -fwd.kron_rotate(GX, np.asarray(R1, np.float64).T, np.asarray(R2, np.float64).T)


def truncate_rank(Y, k: int) -> np.ndarray:
    """Best rank-k approximation in the Frobenius norm (Eckart-Young-Mirsky): truncated SVD."""
    if k <= 0:
        return np.zeros_like(np.asarray(Y, np.float64))
    U, s, Vt = np.linalg.svd(np.asarray(Y, np.float64), full_matrices=False)
    return (U[:, :k] * s[:k]) @ Vt[:k]


def default_mu(s2, n: int, m: int) -> float:
    return 1.0 / (n * m * float(np.min(s2)))


def psp_step(W, M, R1, R2, c, s2, k: int, mu: float | None = None) -> np.ndarray:
    """M_{t+1} = rank-k truncation of M_t - (1 / mu) dL/dM (Sec. 3.2; App. A.2.3)."""
    n, m = np.asarray(W).shape
    if mu is None:
        mu = default_mu(s2, n, m)
    return truncate_rank(np.asarray(M, np.float64) - grad_m(W, M, R1, R2, c, s2) / mu, k)


def factor_low_rank(M, k: int):
    """A = U_k S_k^(1/2), B = S_k^(1/2) V_k^T (App. A.2.3, "a stable choice")."""
    U, s, Vt = np.linalg.svd(np.asarray(M, np.float64), full_matrices=False)
    rs = np.sqrt(s[:k])
    return U[:, :k] * rs, rs[:, None] * Vt[:k]


# --------------------------------------------------------------------------- Algorithm 2
def quantize_layer(W, n1: int, n2: int, k: int, t_outer: int = 5, mu: float | None = None,
                   s2_min: float = S2_MIN, R1=None, R2=None) -> dict:
    """The quantization framework of Algorithm 2 on one weight matrix.  Returns the factors, the
    low-rank pair, the mixture parameters, the final binarization (rows of (W - M) R) and the value
    of L_GMM after every sub-step ("history": list of (outer iteration, step name, value))."""
    W = np.asarray(W, np.float64)
    n, m = W.shape
    assert m == n1 * n2
    R1 = np.eye(n1) if R1 is None else np.asarray(R1, np.float64)
    R2 = np.eye(n2) if R2 is None else np.asarray(R2, np.float64)
    M = np.zeros_like(W)
    c, s2 = init_theta(okt_rows(W, M, R1, R2), s2_min)
    hist = [(-1, "init", gmm_nll(okt_rows(W, M, R1, R2), c, s2))]
    for t in range(t_outer):
        # OKT coordinates and the EM update of the row-wise mixtures
        X = okt_rows(W, M, R1, R2)
        c, s2 = em_step(X, c, s2, s2_min)
        hist.append((t, "em", gmm_nll(X, c, s2)))
        # PSP: proximal step on the low-rank residual
        if k > 0:
            M = psp_step(W, M, R1, R2, c, s2, k, mu)
            hist.append((t, "psp", gmm_nll(okt_rows(W, M, R1, R2), c, s2)))
        # MM: alternating Procrustes updates with targets and weights from the current point
        targets, lam = mm_row_targets(W - M, R1, R2, c, s2)
        R1 = procrustes_r1(W - M, R2, targets, lam, n1, n2)
        targets, lam = mm_row_targets(W - M, R1, R2, c, s2)
        R2 = procrustes_r2(W - M, R1, targets, lam, n1, n2)
        hist.append((t, "mm", gmm_nll(okt_rows(W, M, R1, R2), c, s2)))
    Wrot = fwd.kron_rotate(W - M, R1, R2)
    sgn, alpha, beta = fwd.binarize_rows_centered(Wrot)
    A, B = factor_low_rank(M, k) if k > 0 else (np.zeros((n, 0)), np.zeros((0, m)))
    return dict(R1=R1, R2=R2, M=M, A=A, B=B, c=c, s2=s2, sgn=sgn, alpha=alpha, beta=beta, W_rot=Wrot,
                history=hist)
