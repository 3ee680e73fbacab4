"""Pins of the offline quantizer's oracle (paper App. A.1 Algorithm 2; App. A.2.2; App. A.2.3): every
step is held against something other than its own formula -- a library density, a brute-force grid,
random candidates, finite differences, a dense Kronecker product -- and against the descent
properties the paper states for it.  CPU only."""
import numpy as np
import pytest
import scipy.linalg
import scipy.stats

from oracle import bwla_oracle as fwd
from oracle import bwla_quantizer_oracle as Q


def _rand_orth(rng, n):
    q, r = np.linalg.qr(rng.standard_normal((n, n)))
    return q * np.sign(np.diag(r))


def _problem(seed=0, n=24, n1=4, n2=6, k=2):
    rng = np.random.default_rng(seed)
    W = rng.standard_normal((n, n1 * n2)) * 0.02 + rng.standard_normal((n, 1)) * 0.004
    R1, R2 = _rand_orth(rng, n1), _rand_orth(rng, n2)
    M = Q.truncate_rank(rng.standard_normal(W.shape) * 0.003, k)
    X = Q.okt_rows(W, M, R1, R2)
    c, s2 = Q.init_theta(X)
    return rng, W, M, R1, R2, c, s2


def test_centering_and_okt_rows_are_the_dense_formula():
    """X = (W - M)(R1 (x) R2) H with the dense Kronecker product and the dense H (Sec. 3.2)."""
    rng, W, M, R1, R2, _, _ = _problem()
    m = W.shape[1]
    H = np.eye(m) - np.ones((m, m)) / m
    dense = (W - M) @ np.kron(R1, R2) @ H
    assert np.allclose(Q.okt_rows(W, M, R1, R2), dense, atol=1e-15)
    assert np.allclose(Q.okt_rows(W, M, R1, R2).sum(axis=1), 0.0, atol=1e-15)


def test_nll_and_responsibilities_against_scipy_densities():
    """L_GMM and r^+ written out with scipy.stats.norm.pdf (App. A.2.2, mixture density and E step)."""
    rng, W, M, R1, R2, c, s2 = _problem(1)
    X = Q.okt_rows(W, M, R1, R2)
    sd = np.sqrt(s2)[:, None]
    pp = scipy.stats.norm.pdf(X, loc=c[:, None], scale=sd)
    pm = scipy.stats.norm.pdf(X, loc=-c[:, None], scale=sd)
    assert np.isclose(Q.gmm_nll(X, c, s2), -np.mean(np.log(0.5 * pp + 0.5 * pm)), rtol=1e-12)
    r = Q.responsibilities(X, c, s2)
    assert np.allclose(r, pp / (pp + pm), atol=1e-12)
    assert np.all((r >= 0) & (r <= 1))
    # symmetric in x: r(x) + r(-x) = 1; far tails saturate without overflow
    assert np.allclose(Q.responsibilities(-X, c, s2), 1.0 - r, atol=1e-15)
    far = Q.responsibilities(np.array([[1e6, -1e6]]), np.array([1.0]), np.array([1e-8]))
    assert far[0, 0] == 1.0 and far[0, 1] == 0.0


def test_m_step_maximizes_the_expected_log_likelihood():
    """The closed forms of c_i and s_i^2 against a brute-force grid around them (App. A.2.2, M step)."""
    rng, W, M, R1, R2, c, s2 = _problem(2)
    X = Q.okt_rows(W, M, R1, R2)
    r = Q.responsibilities(X, c, s2)
    cn, sn = Q.m_step(X, r)

    def expected_ll(i, ci, s2i):
        x = X[i]
        return np.sum(r[i] * scipy.stats.norm.logpdf(x, ci, np.sqrt(s2i)) +
                      (1 - r[i]) * scipy.stats.norm.logpdf(x, -ci, np.sqrt(s2i)))
    for i in (0, 5, 17):
        best = expected_ll(i, cn[i], sn[i])
        for fc in (0.9, 0.99, 1.01, 1.1):
            for fs in (0.9, 0.99, 1.0, 1.01, 1.1):
                assert expected_ll(i, cn[i] * fc, sn[i] * fs) <= best + 1e-12
        for fs in (0.9, 0.99, 1.01, 1.1):
            assert expected_ll(i, cn[i], sn[i] * fs) <= best + 1e-12


def test_em_never_increases_the_objective_and_keeps_exact_two_point_rows():
    rng, W, M, R1, R2, c, s2 = _problem(3)
    X = Q.okt_rows(W, M, R1, R2)
    last = Q.gmm_nll(X, c, s2)
    for _ in range(12):
        c, s2 = Q.em_step(X, c, s2)
        now = Q.gmm_nll(X, c, s2)
        assert now <= last + 1e-13
        last = now
    # a row that is exactly +-a: the centre stays at a and the variance falls to its floor
    a = 0.03
    X2 = np.tile(np.array([a, -a, a, -a, a, -a]), (2, 1))
    c2, s22 = Q.em_step(X2, np.array([a, a]), np.array([1e-6, 1e-6]))
    assert np.allclose(c2, a, rtol=1e-12) and np.all(s22 <= 1e-8 + 1e-20)
    # the floor holds
    assert np.all(Q.m_step(X2, Q.responsibilities(X2, c2, s22), s2_min=1e-5)[1] == 1e-5)


def test_quadratic_surrogate_majorizes_the_density_term_and_touches_it():
    """-log p(x') <= (x' - m)^2 / (2 s^2) + const with equality at the point where r, hence m, was taken
    (App. A.2.2, "MM Surrogate"; the paper's surrogate is this without the factor 1/2)."""
    rng = np.random.default_rng(4)
    c, s2 = 0.7, 0.3
    for x0 in (-1.5, -0.2, 0.0, 0.4, 2.0):
        r = Q.responsibilities(np.array([[x0]]), np.array([c]), np.array([s2]))[0, 0]
        m = (2 * r - 1) * c

        def nl(x):
            return -np.log(0.5 * scipy.stats.norm.pdf(x, c, np.sqrt(s2)) + 0.5 * scipy.stats.norm.pdf(x, -c, np.sqrt(s2)))
        const = nl(x0) - (x0 - m) ** 2 / (2 * s2)
        xs = np.concatenate([rng.uniform(-4, 4, 200), [x0]])
        gap = (xs - m) ** 2 / (2 * s2) + const - nl(xs)
        assert np.all(gap >= -1e-12) and abs(gap[-1]) < 1e-12


def test_surrogate_in_kronecker_form_equals_the_dense_one():
    rng, W, M, R1, R2, c, s2 = _problem(5)
    targets, lam = Q.mm_row_targets(W - M, R1, R2, c, s2)
    Y = (W - M) @ np.kron(R1, R2)
    n, m = W.shape
    assert np.isclose(Q.surrogate(W - M, R1, R2, targets, lam), np.sum(lam[:, None] * (Y - targets) ** 2) / (n * m), rtol=1e-13)
    # row by row in the matrix form of App. A.2.2 (this build's convention: R1^T V R2)
    tot = 0.0
    for i in range(n):
        V = (W - M)[i].reshape(R1.shape[0], R2.shape[0])
        tot += lam[i] * np.linalg.norm(R1.T @ V @ R2 - targets[i].reshape(V.shape)) ** 2
    assert np.isclose(tot / (n * m), Q.surrogate(W - M, R1, R2, targets, lam), rtol=1e-13)


def test_row_targets_make_the_surrogate_touch_the_centered_objective():
    """With targets H m_i + mean(y_i) 1 the uncentered quadratic equals the centered one at the
    current factors and lies above it elsewhere (the reading that restores exact descent)."""
    rng, W, M, R1, R2, c, s2 = _problem(6)
    n, m = W.shape
    targets, lam = Q.mm_row_targets(W - M, R1, R2, c, s2)
    m_ij, _ = Q.mm_targets(Q.okt_rows(W, M, R1, R2), c, s2)

    def centered(Ra, Rb):
        X = Q.okt_rows(W, M, Ra, Rb)
        return np.sum(lam[:, None] * (X - Q.center_rows(m_ij)) ** 2) / (n * m)
    assert np.isclose(centered(R1, R2), Q.surrogate(W - M, R1, R2, targets, lam), rtol=1e-12)
    for _ in range(20):
        Ra, Rb = _rand_orth(rng, R1.shape[0]), _rand_orth(rng, R2.shape[0])
        assert centered(Ra, Rb) <= Q.surrogate(W - M, Ra, Rb, targets, lam) + 1e-12


def test_procrustes_updates_against_the_library_and_random_candidates():
    """R1 = U V^T of SVD(C1) is scipy's orthogonal Procrustes solution of the stacked problem, beats
    random orthogonal matrices, and never increases the surrogate (App. A.2.2)."""
    rng, W, M, R1, R2, c, s2 = _problem(7)
    n1, n2 = R1.shape[0], R2.shape[0]
    Wres = W - M
    targets, lam = Q.mm_row_targets(Wres, R1, R2, c, s2)
    s0 = Q.surrogate(Wres, R1, R2, targets, lam)
    R1n = Q.procrustes_r1(Wres, R2, targets, lam, n1, n2)
    assert np.allclose(R1n.T @ R1n, np.eye(n1), atol=1e-13)
    # stacked form: minimize || A R1 - B || with A = [sqrt(lam_i) (V_i R2)^T ...]^T? -- written from
    # R1^T V_i R2 = M_i  <=>  (V_i R2)^T R1 = M_i^T
    V = Wres.reshape(-1, n1, n2)
    A = np.concatenate([np.sqrt(lam[i]) * (V[i] @ R2).T for i in range(len(lam))], axis=0)
    Bm = np.concatenate([np.sqrt(lam[i]) * targets[i].reshape(n1, n2).T for i in range(len(lam))], axis=0)
    Rlib, _ = scipy.linalg.orthogonal_procrustes(A, Bm)
    assert np.allclose(R1n, Rlib, atol=1e-10)
    s1 = Q.surrogate(Wres, R1n, R2, targets, lam)
    assert s1 <= s0 + 1e-15
    for _ in range(50):
        assert s1 <= Q.surrogate(Wres, _rand_orth(rng, n1), R2, targets, lam) + 1e-15
    # second factor: R1^T V_i R2 = M_i  <=>  (R1^T V_i) R2 = M_i
    R2n = Q.procrustes_r2(Wres, R1n, targets, lam, n1, n2)
    A2 = np.concatenate([np.sqrt(lam[i]) * (R1n.T @ V[i]) for i in range(len(lam))], axis=0)
    B2 = np.concatenate([np.sqrt(lam[i]) * targets[i].reshape(n1, n2) for i in range(len(lam))], axis=0)
    R2lib, _ = scipy.linalg.orthogonal_procrustes(A2, B2)
    assert np.allclose(R2n, R2lib, atol=1e-10)
    s2v = Q.surrogate(Wres, R1n, R2n, targets, lam)
    assert s2v <= s1 + 1e-15
    for _ in range(50):
        assert s2v <= Q.surrogate(Wres, R1n, _rand_orth(rng, n2), targets, lam) + 1e-15


def test_mm_step_never_increases_the_true_objective():
    rng, W, M, R1, R2, c, s2 = _problem(8)
    n1, n2 = R1.shape[0], R2.shape[0]
    last = Q.gmm_nll(Q.okt_rows(W, M, R1, R2), c, s2)
    for _ in range(6):
        t, lam = Q.mm_row_targets(W - M, R1, R2, c, s2)
        R1 = Q.procrustes_r1(W - M, R2, t, lam, n1, n2)
        now = Q.gmm_nll(Q.okt_rows(W, M, R1, R2), c, s2)
        assert now <= last + 1e-13
        t, lam = Q.mm_row_targets(W - M, R1, R2, c, s2)
        R2 = Q.procrustes_r2(W - M, R1, t, lam, n1, n2)
        last = Q.gmm_nll(Q.okt_rows(W, M, R1, R2), c, s2)
        assert last <= now + 1e-13


def test_psp_gradient_against_finite_differences():
    """dL(W - M)/dM entry by entry (App. A.2.3, adjoint of T_R; a wrong sign, a missing H or an
    un-transposed factor each fail this)."""
    rng, W, M, R1, R2, c, s2 = _problem(9, n=5, n1=2, n2=3, k=1)
    G = Q.grad_m(W, M, R1, R2, c, s2)
    h = 1e-6
    for (i, j) in ((0, 0), (1, 4), (3, 2), (4, 5)):
        E = np.zeros_like(M)
        E[i, j] = h
        fd = (Q.gmm_nll(Q.okt_rows(W, M + E, R1, R2), c, s2) - Q.gmm_nll(Q.okt_rows(W, M - E, R1, R2), c, s2)) / (2 * h)
        assert np.isclose(G[i, j], fd, rtol=1e-5, atol=1e-9)
    # and the entry-wise gradient in the transformed space
    X = Q.okt_rows(W, M, R1, R2)
    GX = Q.grad_x(X, c, s2)
    E = np.zeros_like(X)
    E[2, 3] = h
    fd = (Q.gmm_nll(X + E, c, s2) - Q.gmm_nll(X - E, c, s2)) / (2 * h)
    assert np.isclose(GX[2, 3], fd, rtol=1e-5, atol=1e-10)


def test_truncated_svd_is_the_best_rank_k_approximation():
    rng = np.random.default_rng(10)
    Y = rng.standard_normal((12, 9))
    for k in (1, 3):
        Mk = Q.truncate_rank(Y, k)
        assert np.linalg.matrix_rank(Mk) == k
        s = np.linalg.svd(Y, compute_uv=False)
        assert np.isclose(np.linalg.norm(Y - Mk) ** 2, np.sum(s[k:] ** 2), rtol=1e-12)      # Eckart-Young-Mirsky
        for _ in range(50):
            cand = rng.standard_normal((12, k)) @ rng.standard_normal((k, 9))
            # best scaling of the candidate, still rank k
            cand *= np.sum(cand * Y) / np.sum(cand * cand)
            assert np.linalg.norm(Y - Mk) <= np.linalg.norm(Y - cand) + 1e-12
        A, B = Q.factor_low_rank(Mk, k)
        assert A.shape == (12, k) and B.shape == (k, 9) and np.allclose(A @ B, Mk, atol=1e-12)
    assert np.all(Q.truncate_rank(Y, 0) == 0)


def test_psp_step_never_increases_the_objective_with_the_default_mu():
    rng, W, M, R1, R2, c, s2 = _problem(11)
    last = Q.gmm_nll(Q.okt_rows(W, M, R1, R2), c, s2)
    for _ in range(8):
        M = Q.psp_step(W, M, R1, R2, c, s2, 2)
        assert np.linalg.matrix_rank(M) <= 2
        now = Q.gmm_nll(Q.okt_rows(W, M, R1, R2), c, s2)
        assert now <= last + 1e-13
        last = now


def test_whole_procedure_descends_and_returns_a_consistent_quantizer():
    """Algorithm 2 on Gaussian rows with a per-row offset: L_GMM after every sub-step is a
    non-increasing sequence, the factors are orthogonal, M = A B has rank k, and the returned
    binarization is the row-wise one of (W - M) R (Sec. 3 "Discussion", Eq. 1-2) -- whose
    dequantized form, taken back through R^T and with M added, approximates W better than the
    plain row-wise binarization of W does."""
    rng = np.random.default_rng(12)
    n, n1, n2, k = 64, 8, 8, 2
    W = rng.standard_normal((n, n1 * n2)) * 0.02 + rng.standard_normal((n, 1)) * 0.005
    out = Q.quantize_layer(W, n1, n2, k, t_outer=6)
    vals = [h[2] for h in out["history"]]
    assert all(b <= a + 1e-12 for a, b in zip(vals, vals[1:])) and vals[-1] < vals[0] - 0.05
    assert [h[1] for h in out["history"][1:4]] == ["em", "psp", "mm"]
    for R in (out["R1"], out["R2"]):
        assert np.allclose(R.T @ R, np.eye(R.shape[0]), atol=1e-12)
    assert np.linalg.matrix_rank(out["M"]) == k and np.allclose(out["A"] @ out["B"], out["M"], atol=1e-12)
    sgn, alpha, beta = fwd.binarize_rows_centered(out["W_rot"])
    assert np.array_equal(sgn, out["sgn"]) and np.array_equal(alpha, out["alpha"]) and np.array_equal(beta, out["beta"])
    assert np.allclose(out["W_rot"], fwd.kron_rotate(W - out["M"], out["R1"], out["R2"]), atol=1e-15)
    deq_rot = out["sgn"] * out["alpha"][:, None] + out["beta"][:, None]
    back = fwd.kron_rotate(deq_rot, out["R1"].T, out["R2"].T) + out["M"]
    s0, a0, b0 = fwd.binarize_rows_centered(W)
    plain = s0 * a0[:, None] + b0[:, None]
    assert np.linalg.norm(W - back) < np.linalg.norm(W - plain)
    # forward equivalence the layer relies on: x W^T = (x R)(W_rot)^T + (x B^T) A^T for the unquantized W_rot
    x = rng.standard_normal((3, n1 * n2))
    assert np.allclose(x @ W.T, fwd.kron_rotate(x, out["R1"], out["R2"]) @ out["W_rot"].T + (x @ out["B"].T) @ out["A"].T,
                       atol=1e-12)


def test_rank_zero_and_identity_start():
    """k = 0: no PSP step appears and M stays zero; the first EM step from the empirical start
    already lowers the objective."""
    rng = np.random.default_rng(13)
    W = rng.standard_normal((16, 24)) * 0.02
    out = Q.quantize_layer(W, 4, 6, 0, t_outer=2)
    assert not np.any(out["M"]) and out["A"].shape == (16, 0)
    assert [h[1] for h in out["history"]] == ["init", "em", "mm", "em", "mm"]
    vals = [h[2] for h in out["history"]]
    assert all(b <= a + 1e-12 for a, b in zip(vals, vals[1:]))
