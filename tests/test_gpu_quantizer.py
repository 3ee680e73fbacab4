"""GPU parity of the offline quantizer (paper App. A.1 Algorithm 2; App. A.2.2; App. A.2.3; Sec. 3.2)
against its fp64 oracle, step by step through the C ABI, on seeded synthetic weight matrices (Gaussian
rows with a row offset and a planted low-rank part: the paper's own matrices are pretrained weights).
Both sides compute in fp64 and differ in summation order only, so the bar is 1e-9 relative on every
step that has a unique result.  The truncated SVD is iterative: with a planted gap behind sigma_k it
is held to 1e-8; without one the singular vectors are not determined to that accuracy by any method,
and the test compares what is unique -- the residual energy (Eckart-Young optimum), the rank, the
singular values -- and the descent of the loss."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import bwla_oracle as fwd
from oracle import bwla_quantizer_oracle as Q

pytestmark = pytest.mark.gpu


def _qb():
    from paper_2605_00422_amd import quantizer_binding as qb
    return qb


def _dev(a, dtype=torch.float64):
    return torch.tensor(np.ascontiguousarray(a), dtype=dtype, device="cuda")


def _rand_orth(rng, n):
    q, r = np.linalg.qr(rng.standard_normal((n, n)))
    return q * np.sign(np.diag(r))


def _problem(seed, n, n1, n2, k, planted=0.0):
    rng = np.random.default_rng(seed)
    m = n1 * n2
    W = rng.standard_normal((n, m)) * 0.02 + rng.standard_normal((n, 1)) * 0.004
    if planted:
        W += planted * (rng.standard_normal((n, k)) @ rng.standard_normal((k, m))) / np.sqrt(k)
    R1, R2 = _rand_orth(rng, n1), _rand_orth(rng, n2)
    U, s, Vt = np.linalg.svd(rng.standard_normal((n, m)) * 0.003, full_matrices=False)
    A, Bt = U[:, :k] * s[:k], Vt[:k].T.copy()
    return rng, W, A, Bt, R1, R2


def _ws(n, m, n1, n2, k):
    return torch.zeros(_qb().workspace_size(n, m, n1, n2, k), dtype=torch.uint8, device="cuda")


def _rel(a, b):
    return float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300))


SHAPES = [(24, 4, 6, 2), (150, 16, 32, 8), (200, 12, 10, 5), (333, 64, 64, 8), (70, 80, 64, 4), (6, 112, 128, 3),
          (10, 86, 64, 3)]


@pytest.mark.parametrize("n,n1,n2,k", SHAPES)
def test_okt_rows_em_and_loss(n, n1, n2, k):
    """X = (W - M) R H, the empirical start, one EM update and L_GMM (Sec. 3.2; App. A.2.2)."""
    qb = _qb()
    _, W, A, Bt, R1, R2 = _problem(1, n, n1, n2, k)
    m = n1 * n2
    ws = _ws(n, m, n1, n2, k)
    X = torch.empty(n, m, dtype=torch.float64, device="cuda")
    ybar = torch.empty(n, dtype=torch.float64, device="cuda")
    qb.okt_rows(_dev(W), _dev(A), _dev(Bt), _dev(R1), _dev(R2), X, ybar, ws)
    M = A @ Bt.T
    Xo = Q.okt_rows(W, M, R1, R2)
    assert _rel(X.cpu().numpy(), Xo) < 1e-11
    assert np.allclose(ybar.cpu().numpy(), fwd.kron_rotate(W - M, R1, R2).mean(axis=1), rtol=1e-9, atol=1e-15)
    # without a low-rank term
    qb.okt_rows(_dev(W), None, None, _dev(R1), _dev(R2), X, None, _ws(n, m, n1, n2, 0))
    assert _rel(X.cpu().numpy(), Q.okt_rows(W, np.zeros_like(W), R1, R2)) < 1e-11
    Xd = _dev(Xo)
    c = torch.empty(n, dtype=torch.float64, device="cuda")
    s2 = torch.empty(n, dtype=torch.float64, device="cuda")
    qb.init_theta(Xd, Q.S2_MIN, c, s2)
    co, s2o = Q.init_theta(Xo)
    assert np.allclose(c.cpu().numpy(), co, rtol=1e-12) and np.allclose(s2.cpu().numpy(), s2o, rtol=1e-11)
    out = torch.empty(1, dtype=torch.float64, device="cuda")
    qb.gmm_nll(Xd, c, s2, out, ws)
    assert abs(out.item() - Q.gmm_nll(Xo, co, s2o)) < 1e-11 * abs(Q.gmm_nll(Xo, co, s2o))
    for _ in range(3):
        qb.em_step(Xd, Q.S2_MIN, c, s2)
        co, s2o = Q.em_step(Xo, co, s2o)
        assert np.allclose(c.cpu().numpy(), co, rtol=1e-10) and np.allclose(s2.cpu().numpy(), s2o, rtol=1e-10)


def test_em_floor_and_degenerate_rows():
    """The variance floor (rows of two exact points +-c) and an all-zero row."""
    qb = _qb()
    n, m = 6, 64
    rng = np.random.default_rng(5)
    X = np.where(rng.random((n, m)) < 0.5, -1.0, 1.0) * 0.25
    X[:, : m // 2] = 0.25
    X[:, m // 2:] = -0.25
    X[3] = 0.0
    Xd = _dev(X)
    c = torch.empty(n, dtype=torch.float64, device="cuda")
    s2 = torch.empty(n, dtype=torch.float64, device="cuda")
    qb.init_theta(Xd, 1e-6, c, s2)
    co, s2o = Q.init_theta(X, 1e-6)
    assert np.array_equal(s2.cpu().numpy(), s2o) and np.all(s2o == 1e-6)
    qb.em_step(Xd, 1e-6, c, s2)
    co, s2o = Q.em_step(X, co, s2o, 1e-6)
    assert np.allclose(c.cpu().numpy(), co, rtol=1e-12, atol=1e-300)
    assert np.allclose(s2.cpu().numpy(), s2o, rtol=1e-12)


@pytest.mark.parametrize("nn", [1, 2, 5, 16, 33, 64, 100, 160, 224, 256])
def test_svd_square_against_lapack(nn):
    """One-sided Jacobi: singular values, orthogonality and the reconstruction G = U S V^T."""
    qb = _qb()
    rng = np.random.default_rng(nn)
    G = rng.standard_normal((nn, nn)) * np.exp(rng.standard_normal((1, nn)))
    sig = torch.empty(nn, dtype=torch.float64, device="cuda")
    Ut = torch.empty(nn, nn, dtype=torch.float64, device="cuda")
    Vt = torch.empty(nn, nn, dtype=torch.float64, device="cuda")
    ws = torch.zeros(2 * nn * nn * 8 + 256, dtype=torch.uint8, device="cuda")
    qb.svd_square(_dev(G), sig, Ut, Vt, ws)
    s, us, v = sig.cpu().numpy(), Ut.cpu().numpy(), Vt.cpu().numpy()
    so = np.linalg.svd(G, compute_uv=False)
    assert np.all(np.diff(s) <= 0)
    assert np.allclose(s, so, rtol=1e-11, atol=1e-13 * so[0])
    assert np.max(np.abs(v @ v.T - np.eye(nn))) < 1e-12
    assert np.max(np.abs(us.T @ v - G)) < 1e-12 * so[0]                     # sum_j (s_j u_j) v_j^T
    u = us / np.maximum(s[:, None], 1e-300)
    assert np.max(np.abs(u @ u.T - np.eye(nn))) < 1e-9


@pytest.mark.parametrize("n,n1,n2,k", SHAPES)
def test_procrustes_updates(n, n1, n2, k):
    """Both Procrustes updates against the oracle's (App. A.2.2); the new factor is orthogonal and
    does not increase the surrogate it minimizes."""
    qb = _qb()
    _, W, A, Bt, R1, R2 = _problem(2, n, n1, n2, k)
    m = n1 * n2
    Wres = W - A @ Bt.T
    c, s2 = Q.init_theta(Q.okt_rows(W, A @ Bt.T, R1, R2))
    c, s2 = Q.em_step(Q.okt_rows(W, A @ Bt.T, R1, R2), c, s2)
    ws = _ws(n, m, n1, n2, 0)
    targets, lam = Q.mm_row_targets(Wres, R1, R2, c, s2)
    for which, nn in ((1, n1), (2, n2)):
        Rn = torch.empty(nn, nn, dtype=torch.float64, device="cuda")
        qb.procrustes(which, _dev(Wres), _dev(R1), _dev(R2), _dev(c), _dev(s2), Rn, ws)
        got = Rn.cpu().numpy()
        want = (Q.procrustes_r1(Wres, R2, targets, lam, n1, n2) if which == 1
                else Q.procrustes_r2(Wres, R1, targets, lam, n1, n2))
        assert np.max(np.abs(got.T @ got - np.eye(nn))) < 1e-12
        assert np.max(np.abs(got - want)) < 1e-9
        before = Q.surrogate(Wres, R1, R2, targets, lam)
        after = Q.surrogate(Wres, got, R2, targets, lam) if which == 1 else Q.surrogate(Wres, R1, got, targets, lam)
        assert after <= before * (1 + 1e-12)


# (the last five: blocks of 80, 128, 132, 160 and 256 vectors -- the Gram matrix's eigenproblem in a row pair of
# lanes per column pair and in a wavefront per pair with the matrix in LDS; above 136 vectors the block is
# orthonormalized by the Newton-Schulz iteration and the eigenproblem is solved once, in scratch)
@pytest.mark.parametrize("n,m,k", [(40, 30, 3), (300, 128, 8), (96, 512, 16), (513, 200, 5), (300, 256, 40),
                                   (400, 300, 64), (300, 280, 66), (400, 320, 80), (500, 300, 128)])
def test_truncate_rank_with_a_gap(n, m, k):
    """Planted rank-k part above a noise floor: the truncation itself is determined, and matches."""
    qb = _qb()
    rng = np.random.default_rng(n + m)
    Y = (rng.standard_normal((n, k)) * np.linspace(3.0, 1.0, k)) @ rng.standard_normal((k, m)) + 0.05 * rng.standard_normal((n, m))
    A = torch.empty(n, k, dtype=torch.float64, device="cuda")
    Bt = torch.empty(m, k, dtype=torch.float64, device="cuda")
    sig = torch.empty(k, dtype=torch.float64, device="cuda")
    ws = torch.zeros(qb.workspace_size(n, m, 1, 1, k), dtype=torch.uint8, device="cuda")
    qb.truncate_rank(_dev(Y), k, 60, 1e-14, A, Bt, sig, ws)
    got = A.cpu().numpy() @ Bt.cpu().numpy().T
    want = Q.truncate_rank(Y, k)
    so = np.linalg.svd(Y, compute_uv=False)
    assert np.allclose(sig.cpu().numpy(), so[:k], rtol=1e-10)
    assert _rel(got, want) < 1e-8
    b = Bt.cpu().numpy()
    assert np.max(np.abs(b.T @ b - np.eye(k))) < 1e-12


def test_truncate_rank_without_a_gap():
    """A Gaussian matrix: what is unique is the residual energy sum_{j>k} sigma_j^2 (Eckart-Young)."""
    qb = _qb()
    n, m, k = 400, 256, 8
    rng = np.random.default_rng(9)
    Y = rng.standard_normal((n, m))
    A = torch.empty(n, k, dtype=torch.float64, device="cuda")
    Bt = torch.empty(m, k, dtype=torch.float64, device="cuda")
    sig = torch.empty(k, dtype=torch.float64, device="cuda")
    ws = torch.zeros(qb.workspace_size(n, m, 1, 1, k), dtype=torch.uint8, device="cuda")
    qb.truncate_rank(_dev(Y), k, 400, 1e-13, A, Bt, sig, ws)
    got = A.cpu().numpy() @ Bt.cpu().numpy().T
    so = np.linalg.svd(Y, compute_uv=False)
    best = float(np.sum(so[k:] ** 2))
    assert np.linalg.matrix_rank(got, tol=1e-9) == k
    res = float(np.sum((Y - got) ** 2))
    assert best * (1 - 1e-12) <= res <= best * (1 + 1e-6)
    assert np.allclose(sig.cpu().numpy(), so[:k], rtol=1e-5)


@pytest.mark.parametrize("n,n1,n2,k", [(150, 16, 32, 8), (333, 64, 64, 8)])
def test_psp_step(n, n1, n2, k):
    """The proximal step with the default mu: the proximal point has a planted low-rank part, so the
    new M matches the oracle's; and L(W - M) does not increase (App. A.2.3)."""
    qb = _qb()
    _, W, A, Bt, R1, R2 = _problem(3, n, n1, n2, k, planted=0.05)
    m = n1 * n2
    M = A @ Bt.T
    X = Q.okt_rows(W, M, R1, R2)
    c, s2 = Q.em_step(X, *Q.init_theta(X))
    Ad, Btd = _dev(A), _dev(Bt)
    qb.psp_step(_dev(W), Ad, Btd, _dev(R1), _dev(R2), _dev(c), _dev(s2), 0.0, 300, 1e-14, _ws(n, m, n1, n2, k))
    got = Ad.cpu().numpy() @ Btd.cpu().numpy().T
    want = Q.psp_step(W, M, R1, R2, c, s2, k)
    before = Q.gmm_nll(X, c, s2)
    after = Q.gmm_nll(Q.okt_rows(W, got, R1, R2), c, s2)
    assert after <= before + 1e-13
    assert abs(after - Q.gmm_nll(Q.okt_rows(W, want, R1, R2), c, s2)) < 1e-9
    # the proximal point and its optimum: residual energy equal to the oracle's
    Yp = M - Q.grad_m(W, M, R1, R2, c, s2) / Q.default_mu(s2, n, m)
    assert np.sum((Yp - got) ** 2) <= np.sum((Yp - want) ** 2) * (1 + 1e-9)
    # an explicit mu goes through the same path
    Ad, Btd = _dev(A), _dev(Bt)
    mu = 3.0 * Q.default_mu(s2, n, m)
    qb.psp_step(_dev(W), Ad, Btd, _dev(R1), _dev(R2), _dev(c), _dev(s2), mu, 300, 1e-14, _ws(n, m, n1, n2, k))
    got = Ad.cpu().numpy() @ Btd.cpu().numpy().T
    want = Q.psp_step(W, M, R1, R2, c, s2, k, mu)
    Yp = M - Q.grad_m(W, M, R1, R2, c, s2) / mu
    assert np.sum((Yp - got) ** 2) <= np.sum((Yp - want) ** 2) * (1 + 1e-9)


@pytest.mark.parametrize("n,n1,n2,k,t", [(150, 16, 32, 4, 3), (256, 32, 32, 0, 3), (333, 64, 64, 8, 2)])
def test_quantize_layer_history_and_outputs(n, n1, n2, k, t):
    """Algorithm 2 end to end: the loss after every sub-step follows the oracle's history and never
    increases; the factors are orthogonal; W_rot = (W - V U^T)(R1 (x) R2); and the result packs and
    runs through the forward path's own pack call."""
    qb = _qb()
    _, W, _, _, _, _ = _problem(4, n, n1, n2, max(k, 1), planted=0.03)
    W = W.astype(np.float32).astype(np.float64)
    m = n1 * n2
    f32 = lambda *s: torch.empty(*s, dtype=torch.float32, device="cuda")
    R1, R2, Wrot = f32(n1, n1), f32(n2, n2), f32(n, m)
    U, V = (f32(m, k), f32(n, k)) if k else (None, None)
    c = torch.empty(n, dtype=torch.float64, device="cuda")
    s2 = torch.empty(n, dtype=torch.float64, device="cuda")
    hist = torch.empty(1 + 3 * t, dtype=torch.float64, device="cuda")
    qb.quantize_layer(_dev(W, torch.float32), n1, n2, k, t, R1, R2, Wrot, U, V, c, s2, hist, _ws(n, m, n1, n2, k),
                      svd_iters=300, svd_tol=1e-14)
    h = hist.cpu().numpy()
    ref = Q.quantize_layer(W, n1, n2, k, t_outer=t)
    want = [v for (_, name, v) in ref["history"]]
    if k == 0:                                            # the oracle records no PSP entry then
        it = iter(want[1:])
        full = [want[0]]
        for _ in range(t):
            em = next(it)
            full += [em, em, next(it)]
        want = full
    assert np.all(np.diff(h) <= 1e-12), h
    assert np.allclose(h, want, rtol=1e-7, atol=1e-9), (h, want)
    r1, r2 = R1.double().cpu().numpy(), R2.double().cpu().numpy()
    assert np.max(np.abs(r1.T @ r1 - np.eye(n1))) < 1e-5 and np.max(np.abs(r2.T @ r2 - np.eye(n2))) < 1e-5
    Mg = V.double().cpu().numpy() @ U.double().cpu().numpy().T if k else np.zeros_like(W)
    wr = Wrot.double().cpu().numpy()
    assert _rel(wr, fwd.kron_rotate(W - Mg, r1, r2)) < 1e-5
    assert abs(Q.gmm_nll(Q.center_rows(wr), c.cpu().numpy(), s2.cpu().numpy()) - h[-1]) < 1e-6
    if k:
        # balanced factors: column norms of V and U agree (both sigma_j^(1/2))
        nv = np.linalg.norm(V.double().cpu().numpy(), axis=0)
        nu = np.linalg.norm(U.double().cpu().numpy(), axis=0)
        assert np.allclose(nv, nu, rtol=1e-5)
    if m % 32 == 0:
        from paper_2605_00422_amd import binding as B
        layer = B.pack_weights(Wrot, R1, R2, U, V, n1, n2, centered=True)
        sgn, alpha = B.unpack_signs(layer)
        so, ao, _ = fwd.binarize_rows_centered(wr)
        assert np.mean(sgn.cpu().numpy() != so) < 1e-3


def test_quantize_layer_at_the_7b_shape():
    """11008 x 4096 (64 x 64), rank 32 -- the shape the benchmark times.  At this size the oracle checks
    what it can compute in seconds: the loss never increases over the sub-steps, the last entry is
    L_GMM of the returned W_rot under the returned mixtures, the factors are orthogonal, and sampled
    rows of W_rot equal (W - V U^T)_i (R1 (x) R2)."""
    qb = _qb()
    n, n1, n2, k, t = 11008, 64, 64, 32, 2
    m = n1 * n2
    rng = np.random.default_rng(7)
    W = (rng.standard_normal((n, m)) * 0.02 + rng.standard_normal((n, 1)) * 0.004).astype(np.float32)
    f32 = lambda *s: torch.empty(*s, dtype=torch.float32, device="cuda")
    R1, R2, Wrot, U, V = f32(n1, n1), f32(n2, n2), f32(n, m), f32(m, k), f32(n, k)
    c = torch.empty(n, dtype=torch.float64, device="cuda")
    s2 = torch.empty(n, dtype=torch.float64, device="cuda")
    hist = torch.empty(1 + 3 * t, dtype=torch.float64, device="cuda")
    qb.quantize_layer(_dev(W, torch.float32), n1, n2, k, t, R1, R2, Wrot, U, V, c, s2, hist, _ws(n, m, n1, n2, k),
                      svd_iters=20, svd_tol=0.0)
    h = hist.cpu().numpy()
    assert np.all(np.isfinite(h)) and np.all(np.diff(h) <= 1e-12), h
    assert h[-1] < h[0] - 1e-3
    r1, r2 = R1.double().cpu().numpy(), R2.double().cpu().numpy()
    assert np.max(np.abs(r1.T @ r1 - np.eye(n1))) < 1e-5 and np.max(np.abs(r2.T @ r2 - np.eye(n2))) < 1e-5
    wr = Wrot.double().cpu().numpy()
    assert abs(Q.gmm_nll(Q.center_rows(wr), c.cpu().numpy(), s2.cpu().numpy()) - h[-1]) < 1e-6
    rows = np.concatenate([[0, n - 1], rng.choice(n, 62, replace=False)])
    Vh, Uh = V.double().cpu().numpy(), U.double().cpu().numpy()
    want = fwd.kron_rotate(W[rows].astype(np.float64) - Vh[rows] @ Uh.T, r1, r2)
    assert _rel(wr[rows], want) < 1e-5
    assert np.linalg.matrix_rank(Vh, tol=1e-9) == k


def test_quantized_layer_through_the_online_path():
    """Algorithm 2's result handed to the online path (Sec. 3.2: Y = Q(X R) B'^T + (X U) V^T): the factors,
    W_rot and the balanced U, V are packed by the forward path's own call and one decode call runs a few
    tokens through them.  The output equals the oracle's forward on the same factors (criterion of
    the parity tests), and against the dense product X W^T it is closer than the layer binarized as it
    stands (identity rotations, no low-rank branch): the planted low-rank part, which dominates the
    binarization error of the raw matrix, now travels through the PSP branch in fp16."""
    from paper_2605_00422_amd import binding as B
    from parity_util import check_output
    qb = _qb()
    n, n1, n2, k, t, M = 512, 32, 32, 8, 3, 8
    m = n1 * n2
    rng, W, _, _, _, _ = _problem(11, n, n1, n2, k, planted=0.05)
    W = W.astype(np.float32).astype(np.float64)
    f32 = lambda *s: torch.empty(*s, dtype=torch.float32, device="cuda")
    R1, R2, Wrot, U, V = f32(n1, n1), f32(n2, n2), f32(n, m), f32(m, k), f32(n, k)
    qb.quantize_layer(_dev(W, torch.float32), n1, n2, k, t, R1, R2, Wrot, U, V, None, None, None, _ws(n, m, n1, n2, k),
                      svd_iters=100, svd_tol=1e-12)
    X = fwd.to_bf16(rng.standard_normal((M, m)))
    Xg = _dev(X, torch.bfloat16)
    dense = X @ W.T

    def run(layer):
        act = B.Activations(layer, M)
        Y = torch.empty((M, n), dtype=torch.float32, device="cuda")
        B.decode_forward(layer, Xg, act, Y)
        torch.cuda.synchronize()
        return Y.double().cpu().numpy()

    Yq = run(B.pack_weights(Wrot, R1, R2, U, V, n1, n2, centered=True))
    ref = fwd.forward(X, R1.double().cpu().numpy(), R2.double().cpu().numpy(), Wrot.double().cpu().numpy(),
                      U.double().cpu().numpy(), V.double().cpu().numpy(), centered=True)
    check_output(Yq, ref["Y"])
    eye = lambda s: torch.eye(s, dtype=torch.float32, device="cuda")
    Y0 = run(B.pack_weights(_dev(W, torch.float32), eye(n1), eye(n2), None, None, n1, n2, centered=True))
    err = lambda Y: float(np.linalg.norm(Y - dense) / np.linalg.norm(dense))
    print(dict(quantized=err(Yq), as_it_stands=err(Y0)), flush=True)
    assert err(Yq) < 0.85 * err(Y0)
