"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test names the passage it rests on.  None of them re-types the oracle's own formula:
they use the dense Kronecker product, invariants, hand-derived values, closed forms,
brute force, and exact special cases.
"""
import math
import os

import numpy as np
import pytest

from oracle import bwla_oracle as orc
from paper_2605_00422_amd import inputs as syn

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    rows = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            rows[parts[0]] = [float(p) for p in parts[1:]]
    return rows


def _orth(rng, n):
    return syn.random_orthogonal(rng, n)


# ------------------------------------------------------------------ Alg. 1 (paper App. A.1)
def test_kron_factor_hand_pairs():
    with open(os.path.join(GOLDEN, "kron_pairs.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            n, n1, n2 = (int(v) for v in line.split())
            assert orc.kron_factor(n) == (n1, n2), n


def test_input_module_pairs_are_algorithm_one():
    """The config table's literal pairs are what Algorithm 1 gives for those widths."""
    for K, pair in syn.KRON_PAIRS.items():
        assert orc.kron_factor(K) == pair, K


def test_kron_factor_properties_bruteforce():
    for n in range(1, 600):
        n1, n2 = orc.kron_factor(n)
        assert n1 * n2 == n and n2 <= n1
        # n2 is the largest divisor not above sqrt(n)
        best = max(d for d in range(1, n + 1) if n % d == 0 and d * d <= n)
        assert n2 == best


# ------------------------------------------------------------------ rotation (paper Sec. 3.1; App. A.2.2)
def test_kron_orthogonal_fp32():
    """R1 (x) R2 is orthogonal: max |Q^T Q - I| < 1e-5 with fp32 factors."""
    rng = np.random.default_rng(1)
    R1, R2 = _orth(rng, 16), _orth(rng, 32)
    Q = np.kron(R1, R2).astype(np.float32)
    assert np.max(np.abs(Q.T @ Q - np.eye(512, dtype=np.float32))) < 1e-5
    # factor-wise for a large K (the dense matrix is never formed there)
    R1, R2 = _orth(rng, 160), _orth(rng, 160)
    for R in (R1, R2):
        assert np.max(np.abs(R.T @ R - np.eye(R.shape[0], dtype=np.float32))) < 1e-5


@pytest.mark.parametrize("n1,n2", [(16, 32), (32, 16), (8, 10), (3, 5), (1, 7), (7, 1)])
def test_rotation_equals_dense_kronecker(n1, n2):
    """The two-small-products form equals X @ kron(R1, R2) (library Kronecker product);
    non-square and n1 != n2 cases catch a swapped factor order or a transposed factor."""
    rng = np.random.default_rng(2)
    R1, R2 = _orth(rng, n1), _orth(rng, n2)
    X = rng.standard_normal((5, n1 * n2))
    ref = X @ np.kron(R1.astype(np.float64), R2.astype(np.float64))
    got = orc.kron_rotate(X, R1, R2)
    assert np.max(np.abs(got - ref)) < 1e-12
    # and the entry-by-entry dense construction agrees with the library one
    assert np.max(np.abs(orc.kron_dense(R1, R2) - np.kron(R1.astype(np.float64), R2.astype(np.float64)))) == 0.0


def test_rotation_not_symmetric_in_factors():
    """Guard for the guard: with n1 != n2 the swapped order really differs."""
    rng = np.random.default_rng(3)
    R1, R2 = _orth(rng, 4), _orth(rng, 6)
    X = rng.standard_normal((2, 24))
    a = X @ np.kron(R1, R2)
    b = X @ np.kron(R2, R1)
    assert np.max(np.abs(a - b)) > 1e-3


def test_rotation_preserves_norm_and_forward_invariance():
    """Orthogonality: ||x R|| = ||x||, and (X R)(W R)^T = X W^T (paper Sec. 1 and 3.1:
    R^-1 = R^T keeps the forward pass unchanged).  Using R^T instead of R on one side
    breaks the second identity."""
    rng = np.random.default_rng(4)
    n1, n2 = 12, 20
    R1, R2 = _orth(rng, n1), _orth(rng, n2)
    X = rng.standard_t(3.0, size=(7, n1 * n2))
    W = rng.standard_normal((9, n1 * n2))
    Xr = orc.kron_rotate(X, R1, R2)
    Wr = orc.kron_rotate(W, R1, R2)
    assert np.allclose(np.linalg.norm(Xr, axis=1), np.linalg.norm(X, axis=1), rtol=1e-6)
    assert np.max(np.abs(Xr @ Wr.T - X @ W.T)) < 1e-4 * np.max(np.abs(X @ W.T))
    # fp32 factors are orthogonal only to ~1e-7, hence the relative bound above; with the
    # wrong direction the mismatch is of order one
    Wbad = orc.kron_rotate(W, R1.T, R2.T)
    assert np.max(np.abs(Xr @ Wbad.T - X @ W.T)) > 1e-2 * np.max(np.abs(X @ W.T))


def test_rotation_identity_factors():
    rng = np.random.default_rng(5)
    X = rng.standard_normal((3, 48))
    assert np.array_equal(orc.kron_rotate(X, np.eye(6), np.eye(8)), X)


# ------------------------------------------------------------------ quantizer (symmetric INT6)
def test_quantizer_range_and_max_maps_to_31():
    rng = np.random.default_rng(6)
    Xr = rng.standard_t(3.0, size=(64, 512))
    q, s, v = orc.quantize_int6(Xr)
    assert q.dtype == np.int8 and q.min() >= -31 and q.max() <= 31
    for t in range(Xr.shape[0]):
        k = int(np.argmax(np.abs(Xr[t])))
        assert abs(int(q[t, k])) == 31 and np.sign(q[t, k]) == np.sign(Xr[t, k])
        assert np.max(np.abs(q[t])) == 31
    # reconstruction error is at most half a step everywhere
    assert np.max(np.abs(q * s[:, None] - Xr) / s[:, None]) <= 0.5 + 1e-12


def test_quantizer_integer_input_is_reproduced():
    """Integer-valued X~ with amax 31 gives q = X~ and s = 1 exactly."""
    rng = np.random.default_rng(7)
    Xr = rng.integers(-31, 32, size=(8, 96)).astype(np.float64)
    Xr[:, 0] = 31.0
    q, s, _ = orc.quantize_int6(Xr)
    assert np.array_equal(q.astype(np.float64), Xr) and np.all(s == 1.0)


def test_quantizer_ties_to_even_zero_token_and_scale_equivariance():
    # amax = 31 so v = x: ties at .5 go to the even neighbour
    Xr = np.array([[31.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 30.5]])
    q, s, v = orc.quantize_int6(Xr)
    assert q.tolist() == [[31, 0, 2, 2, 0, -2, -2, 30]]
    q0, s0, v0 = orc.quantize_int6(np.zeros((2, 8)))
    assert not q0.any() and not s0.any() and not v0.any()
    # scaling a token by a power of two changes s, not q
    rng = np.random.default_rng(8)
    A = rng.standard_normal((4, 64))
    qa, sa, _ = orc.quantize_int6(A)
    qb, sb, _ = orc.quantize_int6(A * 8.0)
    assert np.array_equal(qa, qb) and np.allclose(sb, 8.0 * sa, rtol=0, atol=0)
    # negation flips the codes
    qc, _, _ = orc.quantize_int6(-A)
    assert np.array_equal(qc, -qa)


@pytest.mark.parametrize("bits,qmax", [(4, 7), (6, 31), (8, 127)])
def test_quantizer_other_widths(bits, qmax):
    """The same quantizer at 4, 6 and 8 bits: range, the maximum maps to +-qmax with its sign,
    half-step reconstruction bound, integer inputs reproduced, ties to even, and agreement with a
    scalar loop (Python's round is half-to-even)."""
    rng = np.random.default_rng(30 + bits)
    Xr = rng.standard_t(3.0, size=(16, 96))
    q, s, v = orc.quantize_sym(Xr, bits)
    assert q.dtype == np.int8 and q.min() >= -qmax and q.max() <= qmax
    for t in range(Xr.shape[0]):
        k = int(np.argmax(np.abs(Xr[t])))
        assert int(q[t, k]) == qmax * int(np.sign(Xr[t, k]))
        amax = max(abs(float(x)) for x in Xr[t])
        assert math.isclose(s[t], amax / qmax, rel_tol=1e-15)
        assert q[t].tolist() == [max(-qmax, min(qmax, round(qmax * float(x) / amax))) for x in Xr[t]]
    assert np.max(np.abs(q * s[:, None] - Xr) / s[:, None]) <= 0.5 + 1e-12
    Xi = rng.integers(-qmax, qmax + 1, size=(4, 40)).astype(np.float64)
    Xi[:, 1] = -qmax
    qi, si, _ = orc.quantize_sym(Xi, bits)
    assert np.array_equal(qi.astype(np.float64), Xi) and np.all(si == 1.0)
    tie = np.array([[float(qmax), 0.5, 1.5, 2.5, -0.5, -1.5, -2.5]])
    assert orc.quantize_sym(tie, bits)[0].tolist() == [[qmax, 0, 2, 2, 0, -2, -2]]
    if bits == 6:
        a, b = orc.quantize_int6(Xr), (q, s, v)
        assert all(np.array_equal(x, y) for x, y in zip(a, b))
    with pytest.raises(ValueError):
        orc.quantize_sym(Xr, 9)


def test_forward_with_eight_bit_codes_is_closer_to_the_unquantized_layer():
    """Finer activation codes can only help: the same layer at 4, 6 and 8 bits against the
    rotated, binarized layer applied to unquantized activations."""
    cfg = syn.CONFIGS["cfg0_tiny"]
    d = syn.make_layer(cfg)
    sgn, alpha = orc.binarize_rows(d.W)
    exact = orc.kron_rotate(d.X, d.R1, d.R2) @ (orc.to_fp16(alpha)[:, None] * sgn).T + orc.psp_project(d.X, d.U) @ d.V.astype(np.float64).T
    err = [np.linalg.norm(orc.forward(d.X, d.R1, d.R2, d.W, d.U, d.V, act_bits=b)["Y"] - exact) for b in (4, 6, 8)]
    assert err[0] > 2.5 * err[1] > 2.5 * 2.5 * err[2] > 0


# ------------------------------------------------------------------ asymmetric activation codes
@pytest.mark.parametrize("bits", [4, 6, 8])
def test_asymmetric_quantizer_against_scalar_loop_and_invariants(bits):
    L = (1 << bits) - 1
    rng = np.random.default_rng(40 + bits)
    Xr = rng.standard_t(3.0, size=(12, 80)) + rng.normal(0.0, 2.0, size=(12, 1))     # skewed tokens
    Xr[3] = np.abs(Xr[3])                                   # a token without negative values: lo = 0
    Xr[4] = -np.abs(Xr[4])                                  # and one without positive values: hi = 0
    q, s, z, v, u = orc.quantize_asym(Xr, bits)
    assert q.min() >= 0 and q.max() <= L and z.min() >= 0 and z.max() <= L
    for t in range(Xr.shape[0]):
        lo = min(min(float(x) for x in Xr[t]), 0.0)
        hi = max(max(float(x) for x in Xr[t]), 0.0)
        st = (hi - lo) / L
        zt = round(-lo / st)                                # Python's round: half to even
        assert math.isclose(s[t], st, rel_tol=1e-15) and z[t] == zt
        assert q[t].tolist() == [max(0, min(L, round(float(x) / st) + zt)) for x in Xr[t]]
        # the ends of the range land on the ends of the code range (up to the rounding of z), zero is exact
        assert q[t, int(np.argmin(Xr[t]))] <= 1 or lo == 0.0
        assert q[t, int(np.argmax(Xr[t]))] >= L - 1 or hi == 0.0
    assert z[3] == 0 and z[4] == L
    # reconstruction: half a step inside the range; one step more where the rounding of z moved the range
    rec = s[:, None] * (q - z[:, None])
    assert np.max(np.abs(rec - Xr) / s[:, None]) <= 1.0 + 1e-9
    inner = (q > 0) & (q < L)
    assert np.max((np.abs(rec - Xr) / s[:, None])[inner]) <= 0.5 + 1e-9
    zero = orc.quantize_asym(np.zeros((2, 8)), bits)
    assert not zero[0].any() and not zero[1].any() and not zero[2].any()
    # a token that is symmetric about zero has its zero point in the middle
    sym = np.array([[-3.0, -1.0, 0.0, 1.0, 3.0]])
    assert orc.quantize_asym(sym, bits)[2][0] in ((L - 1) // 2, (L + 1) // 2)


def test_asymmetric_codes_integer_case_is_exact():
    """Tokens whose values are integers spanning exactly [lo, lo + 63]: s = 1, z = -lo, q - z = X~."""
    rng = np.random.default_rng(44)
    Xr = rng.integers(-20, 44, size=(5, 64)).astype(np.float64)
    Xr[:, 0], Xr[:, 1] = -20.0, 43.0
    q, s, z, v, u = orc.quantize_asym(Xr, 6)
    assert np.all(s == 1.0) and np.all(z == 20)
    assert np.array_equal(q - z[:, None], Xr.astype(np.int64))


def test_asymmetric_forward_equals_dense_dequantized_product_and_loops():
    rng = np.random.default_rng(45)
    n1, n2, N, r, M = 4, 8, 7, 3, 5
    K = n1 * n2
    X = rng.standard_t(3.0, size=(M, K)) + 0.7
    R1, R2 = _orth(rng, n1), _orth(rng, n2)
    W = rng.normal(0.05, 0.3, size=(N, K))
    U = orc.to_fp16(rng.normal(size=(K, r)) * 0.1); V = orc.to_fp16(rng.normal(size=(N, r)) * 0.1)
    for centered in (False, True):
        out = orc.forward_asym(X, R1, R2, W, U, V, centered=centered)
        # dense route: dequantized activations times dequantized weights
        xhat = out["s"][:, None] * (out["q"] - out["z"][:, None])
        Wdeq = out["alpha16"][:, None] * out["sgn"] + (orc.to_fp16(out["mu"])[:, None] if centered else 0.0)
        Yd = xhat @ Wdeq.T + (X @ U) @ V.T
        assert np.allclose(out["Y"], Yd, rtol=1e-12, atol=1e-12)
        # the contraction as a literal loop over Python ints
        for t in range(M):
            for n in range(N):
                a = sum(int(out["c"][t, k]) * int(out["sgn"][n, k]) for k in range(K))
                assert a == out["acc_c"][t, n]
    # what the GPU uses: codes stored with an offset, q' = q - 32, z' = z - 32, and the zero point
    # taken out of the accumulator as a rank-one term  sum_k (q - z) sgn = sum_k q' sgn - z' rowsum
    out = orc.forward_asym(X, R1, R2, W, U, V)
    qp = out["q"].astype(np.int64) - 32
    zp = out["z"] - 32
    rowsum = out["sgn"].astype(np.int64).sum(axis=1)
    assert np.array_equal(orc.binary_gemm(qp.astype(np.int8), out["sgn"]) - zp[:, None] * rowsum[None, :], out["acc_c"])


def test_asymmetric_beats_symmetric_on_skewed_tokens_and_matches_it_in_accuracy_on_symmetric_ones():
    rng = np.random.default_rng(46)
    cfg = syn.CONFIGS["cfg0_tiny"]
    d = syn.make_layer(cfg)
    sgn, alpha = orc.binarize_rows(d.W)
    Wb = orc.to_fp16(alpha)[:, None] * sgn
    low = orc.psp_project(d.X, d.U) @ d.V.astype(np.float64).T
    exact = orc.kron_rotate(d.X, d.R1, d.R2) @ Wb.T + low
    e_sym = np.linalg.norm(orc.forward(d.X, d.R1, d.R2, d.W, d.U, d.V)["Y"] - exact)
    e_asym = np.linalg.norm(orc.forward_asym(d.X, d.R1, d.R2, d.W, d.U, d.V)["Y"] - exact)
    assert 0.3 * e_sym < e_asym < 1.2 * e_sym               # same step size up to the spare level: same accuracy class
    # a rotated token with a large offset: the symmetric range wastes half of its codes
    Xr = rng.normal(5.0, 1.0, size=(8, 256))
    qs, ss, _ = orc.quantize_sym(Xr, 6)
    qa, sa, za, _, _ = orc.quantize_asym(Xr, 6)
    err_s = np.linalg.norm(qs * ss[:, None] - Xr)
    err_a = np.linalg.norm(sa[:, None] * (qa - za[:, None]) - Xr)
    assert err_a < 0.6 * err_s


# ------------------------------------------------------------------ binarization (paper Eq. 1-4; App. A.2.4)
def test_sign_convention_zero_is_minus_one():
    sgn, alpha = orc.binarize_rows(np.array([[0.0, 1e-30, -1e-30, 2.0]]))
    assert sgn.tolist() == [[-1, 1, -1, 1]]


def test_alpha_is_the_least_squares_scale_with_variance_residual():
    """alpha* = mean |w| minimizes sum (w - alpha sign(w))^2 and the minimum is
    K Var(|w|) (paper App. A.2.4)."""
    rng = np.random.default_rng(9)
    W = rng.standard_normal((6, 200)) * 0.02
    sgn, alpha = orc.binarize_rows(W)
    for i in range(W.shape[0]):
        err = lambda a: float(np.sum((W[i] - a * sgn[i]) ** 2))
        e0 = err(alpha[i])
        assert e0 <= err(alpha[i] * 1.001) and e0 <= err(alpha[i] * 0.999)
        grid = np.linspace(0, 0.1, 2001)
        assert abs(grid[np.argmin([err(a) for a in grid])] - alpha[i]) <= 1e-4
        assert math.isclose(e0, W.shape[1] * np.var(np.abs(W[i])), rel_tol=1e-10)


def test_two_point_rows_are_recovered_exactly():
    """A row with values in {+c, -c} is reproduced exactly by sign * alpha (App. A.2.4)."""
    rng = np.random.default_rng(10)
    c = np.array([0.5, 0.03125, 2.0])
    S = np.where(rng.random((3, 64)) > 0.5, 1.0, -1.0)
    W = S * c[:, None]
    sgn, alpha = orc.binarize_rows(W)
    assert np.array_equal(sgn * alpha[:, None], W)


def test_binarized_layer_bruteforce_tiny():
    """Brute force: y[n] = sum_k x[k] * (w[n,k] > 0 ? +alpha_n : -alpha_n) by scalar loops."""
    rng = np.random.default_rng(11)
    W = rng.standard_normal((5, 12))
    q = rng.integers(-31, 32, size=(3, 12)).astype(np.int8)
    sgn, alpha = orc.binarize_rows(W)
    acc = orc.binary_gemm(q, sgn)
    for t in range(3):
        for n in range(5):
            a = sum(abs(W[n, k]) for k in range(12)) / 12
            ref = sum(int(q[t, k]) * (a if W[n, k] > 0 else -a) for k in range(12))
            assert math.isclose(alpha[n] * acc[t, n], ref, rel_tol=1e-12, abs_tol=1e-12)


# ------------------------------------------------------------------ integer GEMM
def test_binary_gemm_matches_triple_loop_and_bound():
    rng = np.random.default_rng(12)
    q = rng.integers(-31, 32, size=(16, 512)).astype(np.int8)
    sgn = np.where(rng.random((40, 512)) > 0.5, 1, -1).astype(np.int8)
    a = orc.binary_gemm(q, sgn)
    b = orc.binary_gemm_loops(q.tolist(), sgn.tolist())
    assert a.dtype == np.int64 and np.array_equal(a, b)
    assert np.max(np.abs(a)) <= 31 * 512
    # extreme: all codes 31, all signs +1 reaches the bound exactly
    assert orc.binary_gemm(np.full((1, 64), 31, np.int8), np.ones((1, 64), np.int8))[0, 0] == 31 * 64


# ------------------------------------------------------------------ PSP branch (paper Sec. 3.2)
def test_low_rank_split_is_function_preserving():
    """x (W - V U^T)^T + (x U) V^T = x W^T: adding the branch restores the layer."""
    rng = np.random.default_rng(13)
    X = rng.standard_normal((4, 30))
    W = rng.standard_normal((7, 30))
    U = rng.standard_normal((30, 3))
    V = rng.standard_normal((7, 3))
    T = orc.psp_project(X, U)
    lhs = X @ (W - V @ U.T).T + orc.dequant_output(np.zeros((4, 7)), np.ones(4), np.ones(7), T, V)
    assert np.max(np.abs(lhs - X @ W.T)) < 1e-12
    assert T.shape == (4, 3)
    # a transposed or swapped factor cannot satisfy this with these shapes (7 != 30 != 3)


# ------------------------------------------------------------------ binarization with the row shift
def test_centered_binarization_matches_scalar_loops_and_sign_of_zero():
    rng = np.random.default_rng(21)
    W = rng.normal(0.3, 1.0, size=(5, 12))
    W[2, :] = [1.0, 3.0, 1.0, 3.0, 2.0, 2.0, 1.0, 3.0, 2.0, 2.0, 1.0, 3.0]   # mean 2: four exact zeros after centering
    sgn, delta, mu = orc.binarize_rows_centered(W)
    for n in range(5):
        m = math.fsum(W[n]) / 12
        assert math.isclose(mu[n], m, rel_tol=1e-15, abs_tol=1e-16)
        assert math.isclose(delta[n], math.fsum(abs(w - m) for w in W[n]) / 12, rel_tol=1e-14)
    assert mu[2] == 2.0 and math.isclose(delta[2], 2.0 / 3.0, rel_tol=1e-15)
    assert sgn[2].tolist() == [-1, 1, -1, 1, -1, -1, -1, 1, -1, -1, -1, 1]    # Sign(0) = -1
    assert np.array_equal(sgn[[0, 1, 3, 4]], np.where(W[[0, 1, 3, 4]] - mu[[0, 1, 3, 4], None] > 0, 1, -1))


def test_centered_scale_is_least_squares_and_shifted_two_point_rows_are_exact():
    rng = np.random.default_rng(22)
    W = rng.normal(-0.2, 0.5, size=(4, 64))
    sgn, delta, mu = orc.binarize_rows_centered(W)
    C = W - mu[:, None]
    loss = lambda d: np.sum((C - d[:, None] * sgn) ** 2, axis=1)
    base = loss(delta)
    assert np.allclose(base, 64 * np.var(np.abs(C), axis=1), rtol=1e-12)      # K * Var|w - mu|
    for eps in (1e-3, -1e-3):
        assert np.all(loss(delta + eps) > base)
    # rows that take the two values mu +- c equally often are reproduced exactly
    c = np.array([0.5, 0.125, 2.0]); m = np.array([1.0, -0.25, 4.0])
    pat = np.tile([1.0, -1.0], 8)
    W2 = m[:, None] + c[:, None] * np.stack([pat, np.roll(pat, 1), pat])
    sgn2, delta2, mu2 = orc.binarize_rows_centered(W2)
    assert np.array_equal(mu2, m) and np.array_equal(delta2, c)
    assert np.array_equal(delta2[:, None] * sgn2 + mu2[:, None], W2)


def test_centered_dequantization_is_the_product_with_the_dequantized_weights():
    """Y = s (delta acc + mu qsum) + T V^T against the dense route: dequantized activations
    times W_deq = delta sgn + mu (paper Eq. 4), plus the low-rank product."""
    rng = np.random.default_rng(23)
    M, K, N, r = 7, 48, 9, 3
    q = rng.integers(-31, 32, size=(M, K)).astype(np.int8)
    s = rng.uniform(0.01, 0.2, size=M)
    W = rng.normal(0.1, 0.3, size=(N, K))
    sgn, delta, mu = orc.binarize_rows_centered(W)
    T = rng.normal(size=(M, r)); V = rng.normal(size=(N, r))
    acc = orc.binary_gemm(q, sgn)
    Y = orc.dequant_output_centered(acc, s, delta, mu, q.astype(np.int64).sum(axis=1), T, V)
    Wdeq = delta[:, None] * sgn + mu[:, None]
    Yd = (s[:, None] * q.astype(np.float64)) @ Wdeq.T + T @ V.T
    assert np.allclose(Y, Yd, rtol=1e-12, atol=1e-12)
    # dropping the shift term is a different result (the term is really there)
    assert not np.allclose(orc.dequant_output(acc, s, delta, T, V), Yd, rtol=1e-3)


def test_centered_equals_uncentered_when_row_means_vanish():
    rng = np.random.default_rng(24)
    n1, n2, N = 4, 8, 6
    half = rng.integers(-60, 61, size=(N, 16)) / 1024.0       # dyadic grid: every partial sum is exact
    W = np.concatenate([half, -half], axis=1)                 # every row sums to zero exactly
    W = W[:, rng.permutation(32)]
    X = rng.standard_t(3, size=(5, 32))
    R1, R2 = _orth(rng, n1), _orth(rng, n2)
    a = orc.forward(X, R1, R2, W)
    b = orc.forward(X, R1, R2, W, centered=True)
    assert np.array_equal(b["mu"], np.zeros(N))
    assert np.array_equal(a["sgn"], b["sgn"]) and np.array_equal(a["alpha16"], b["alpha16"])
    assert np.allclose(a["Y"], b["Y"], rtol=1e-14, atol=0.0)  # (same value, products taken in another order)


def test_hand_example_centered():
    g = _read_golden("hand_example_centered.txt")
    X = np.array([g["x"]])
    R1 = np.array(g["R1"]).reshape(2, 2)
    R2 = np.array(g["R2"]).reshape(2, 2)
    W = np.array([g["w0"], g["w1"]])
    out = orc.forward(X, R1, R2, W, centered=True)
    assert out["q"][0].tolist() == [int(v) for v in g["q"]]
    assert math.isclose(out["s"][0], g["s"][0], rel_tol=1e-15)
    assert out["mu"].tolist() == g["mu"] and out["alpha"].tolist() == g["delta"]
    assert out["sgn"].tolist() == [[int(v) for v in g["sgn0"]], [int(v) for v in g["sgn1"]]]
    Wdeq = out["alpha"][:, None] * out["sgn"] + out["mu"][:, None]
    assert Wdeq.tolist() == [g["wdeq0"], g["wdeq1"]]
    assert out["acc"][0].tolist() == [int(v) for v in g["acc"]]
    assert out["qsum"][0] == int(g["qsum"][0])
    assert np.allclose(out["Y"][0], g["y"], rtol=1e-14)


def test_centered_forward_rows_matches_forward():
    rng = np.random.default_rng(25)
    cfg = syn.CONFIGS["cfg0_tiny"]
    d = syn.make_layer(cfg)
    W = d.W + rng.normal(0.0, 0.01, size=(cfg.N, 1)).astype(np.float32)
    full = orc.forward(d.X, d.R1, d.R2, W, d.U, d.V, centered=True)
    sgn, delta, mu = orc.binarize_rows_centered(W)
    rows = np.array([0, 5, 15])
    part = orc.forward_rows(d.X, d.R1, d.R2, sgn, orc.to_fp16(delta), d.U, d.V, rows, mu16=orc.to_fp16(mu))
    assert np.array_equal(part["Y"], full["Y"][rows]) and np.array_equal(part["q"], full["q"][rows])
    # and the shift matters at this size: without it the output moves by more than the tolerance
    plain = orc.forward_rows(d.X, d.R1, d.R2, sgn, orc.to_fp16(delta), d.U, d.V, rows)
    assert np.linalg.norm(plain["Y"] - part["Y"]) > 1e-2 * np.linalg.norm(part["Y"])


# ------------------------------------------------------------------ end to end
def test_hand_example_2x2():
    g = _read_golden("hand_example_2x2.txt")
    X = np.array([g["x"]])
    R1 = np.array(g["R1"]).reshape(2, 2)
    R2 = np.array(g["R2"]).reshape(2, 2)
    W = np.array([g["w0"], g["w1"]])
    out = orc.forward(X, R1, R2, W)
    assert np.allclose(out["Xr"][0], g["xr"], atol=1e-14)
    assert out["q"][0].tolist() == [int(v) for v in g["q"]]
    assert math.isclose(out["s"][0], g["s"][0], rel_tol=1e-15)
    assert out["sgn"].tolist() == [[int(v) for v in g["sgn0"]], [int(v) for v in g["sgn1"]]]
    assert out["alpha"].tolist() == g["alpha"]
    assert out["acc"][0].tolist() == [int(v) for v in g["acc"]]
    assert np.allclose(out["Y"][0], g["y"], rtol=1e-14)
    assert out["qsum"][0] == sum(int(v) for v in g["q"])


def test_exact_case_identity_rotation_rank0():
    """R = I, r = 0, integer X with amax 31, W in {+c,-c} with c on the fp16 grid:
    the quantized path equals the plain product X W^T exactly, which is also the plain
    sign-weight GEMM."""
    rng = np.random.default_rng(14)
    n1, n2, N = 4, 8, 10
    X = rng.integers(-31, 32, size=(6, n1 * n2)).astype(np.float64)
    X[:, 3] = -31.0
    c = 2.0 ** rng.integers(-6, 2, size=N)
    W = np.where(rng.random((N, n1 * n2)) > 0.5, 1.0, -1.0) * c[:, None]
    out = orc.forward(X, np.eye(n1), np.eye(n2), W)
    assert np.array_equal(out["Y"], X @ W.T)
    assert np.array_equal(out["acc"], (X @ np.sign(W).T).astype(np.int64))


def test_full_path_equals_scalar_loops_tiny():
    """The vectorized oracle equals the all-scalar dense-definition loops."""
    cfg = syn.LayerConfig("t", 3, 24, 4, 6, 5, 2, "f32", 2, 20.0, seed=3)
    d = syn.make_layer(cfg)
    out = orc.forward(d.X, d.R1, d.R2, d.W, d.U, d.V)
    ref = orc.forward_loops(d.X, d.R1, d.R2, d.W, d.U, d.V)
    assert np.max(np.abs(out["Y"] - ref)) <= 1e-12 * np.max(np.abs(ref))


def test_forward_rows_matches_forward():
    cfg = syn.LayerConfig("t", 9, 64, 8, 8, 12, 4, "bf16", 2, 20.0, seed=5)
    d = syn.make_layer(cfg)
    full = orc.forward(d.X, d.R1, d.R2, d.W, d.U, d.V)
    rows = np.array([0, 4, 8])
    sub = orc.forward_rows(d.X, d.R1, d.R2, full["sgn"], full["alpha16"], d.U, d.V, rows)
    assert np.array_equal(sub["q"], full["q"][rows])
    assert np.array_equal(sub["acc"], full["acc"][rows])
    assert np.array_equal(sub["Y"], full["Y"][rows])


def test_quantized_path_tracks_the_unquantized_layer():
    """Sanity of the approximation (not a pin of its accuracy): with R = identity the output
    correlates strongly with x (sign(W) alpha)^T."""
    cfg = syn.LayerConfig("t", 8, 512, 16, 32, 64, 8, "f32", 0, 1.0, seed=7)
    d = syn.make_layer(cfg)
    out = orc.forward(d.X, d.R1, d.R2, d.W, d.U, d.V)
    Xr = orc.kron_rotate(d.X, d.R1, d.R2)
    ref = Xr @ (out["sgn"] * out["alpha16"][:, None]).T + (d.X.astype(np.float64) @ d.U) @ d.V.T
    rel = np.linalg.norm(out["Y"] - ref) / np.linalg.norm(ref)
    assert rel < 0.05


# ------------------------------------------------------------------ storage accounting (paper Table 1)
def test_swiglu_hand_values_identities_and_interleaving():
    """silu at hand-computed points, its odd-part identity silu(x) - silu(-x) = x, its limits, the
    order of the two operands (gate goes through silu, up does not) and the column interleaving."""
    Y = np.array([[1.0, 1.0, 2.0, 3.0, 3.0, 2.0, 0.0, 5.0, -1.0, 4.0]])
    h = orc.swiglu_interleaved(Y)
    assert h.shape == (1, 5)
    e = math.e
    want = [1.0 / (1.0 + 1.0 / e), 2.0 / (1.0 + e ** -2) * 3.0, 3.0 / (1.0 + e ** -3) * 2.0, 0.0,
            -1.0 / (1.0 + e) * 4.0]
    assert np.allclose(h[0], want, rtol=1e-15, atol=0)
    assert abs(h[0, 0] - 0.7310585786300049) < 1e-15          # silu(1), tabulated logistic value
    assert abs(h[0, 1] - h[0, 2]) > 0.4                       # swapping gate and up changes the result
    x = np.linspace(-30, 30, 241)
    silu = lambda v: orc.swiglu_interleaved(np.stack([v, np.ones_like(v)], axis=1).reshape(1, -1))[0]
    assert np.allclose(silu(x) - silu(-x), x, rtol=0, atol=1e-13)
    assert np.allclose(silu(np.array([40.0, 700.0])), [40.0, 700.0], rtol=1e-15)
    assert np.all(np.abs(silu(np.array([-40.0, -700.0, -800.0]))) < 1e-15)   # exp overflows to inf: -0
    # minimum of silu: at x0 with x0 + 1 + exp(-x0)... = 0, value about -0.27846
    assert abs(silu(x).min() - (-0.2784645)) < 1e-4
    # linear in the up operand
    Y2 = Y.copy(); Y2[:, 1::2] *= -2.5
    assert np.allclose(orc.swiglu_interleaved(Y2), -2.5 * h, rtol=1e-15)


def test_to_bf16_rounds_to_nearest_even_on_eight_bits():
    """bfloat16 keeps 8 significant bits: spot values around 1 (spacing 2^-7), ties to even, and
    agreement with the input generator's fp32 bit trick on fp32-representable values."""
    u = 2.0 ** -7
    vals = np.array([1.0, 1.0 + u, 1.0 + 0.5 * u, 1.0 + 1.5 * u, 1.0 + 0.49 * u, 1.0 + 0.51 * u, -3.0 - 2 * u, 0.0])
    want = np.array([1.0, 1.0 + u, 1.0, 1.0 + 2 * u, 1.0, 1.0 + u, -3.0 - 2 * u, 0.0])
    assert np.array_equal(orc.to_bf16(vals), want)
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(5000) * np.exp(rng.uniform(-20, 20, 5000))).astype(np.float32)
    assert np.array_equal(orc.to_bf16(x.astype(np.float64)), syn.round_to_bf16(x).astype(np.float64))
    # a value that double rounding (fp64 -> fp32 -> bf16) would get wrong: just above a bf16 tie,
    # by less than half an fp32 ulp
    t = 1.0 + 0.5 * u + 2.0 ** -30
    assert orc.to_bf16(np.array([t]))[0] == 1.0 + u
    assert syn.round_to_bf16(np.array([t], dtype=np.float32))[0] == 1.0


def test_to_fp16_rounds_to_nearest_even_on_eleven_bits():
    """fp16 keeps 11 significant bits (spacing 2^-10 in [1, 2)), has subnormals of 2^-24 below 2^-14
    and overflows to infinity from 65520 on: spot values and ties, a value that double rounding
    through fp32 gets wrong, and exact rational arithmetic on random values of every binade."""
    from fractions import Fraction
    u = 2.0 ** -10
    vals = np.array([1.0, 1.0 + u, 1.0 + 0.5 * u, 1.0 + 1.5 * u, 1.0 + 0.49 * u, 1.0 + 0.51 * u, -3.0 - 2 * u, 0.0,
                     65504.0, 65519.9, 2.0 ** -24, 0.5 * 2.0 ** -24, 1.5 * 2.0 ** -24, 2.0 ** -14 - 2.0 ** -25])
    want = np.array([1.0, 1.0 + u, 1.0, 1.0 + 2 * u, 1.0, 1.0 + u, -3.0 - 2 * u, 0.0,
                     65504.0, 65504.0, 2.0 ** -24, 0.0, 2.0 ** -23, 2.0 ** -14])
    assert np.array_equal(orc.to_fp16(vals), want)
    with np.errstate(over="ignore"):
        assert np.isinf(orc.to_fp16(np.array([65520.0]))[0])
    # just above a tie by less than half an fp32 ulp: fp64 -> fp32 lands on the tie, which then goes to even
    t = 1.0 + 0.5 * u + 2.0 ** -30
    assert orc.to_fp16(np.array([t]))[0] == 1.0 + u
    assert np.float16(np.float32(t)) == np.float16(1.0)

    def rational(x):
        f = Fraction(x)
        if f == 0:
            return 0.0
        e = math.floor(math.log2(abs(x)))
        while Fraction(2) ** e > abs(f):
            e -= 1
        while Fraction(2) ** (e + 1) <= abs(f):
            e += 1
        quantum = Fraction(2) ** (max(e, -14) - 10)
        return float(round(f / quantum) * quantum)      # Python rounds a Fraction half to even

    rng = np.random.default_rng(11)
    x = rng.standard_normal(4000) * np.exp2(rng.uniform(-27, 15.9, 4000))
    # scales and factors as the layers store them: |w| ~ 0.016, U and V ~ 0.01
    x = np.concatenate([x, rng.standard_normal(2000) * 0.01, np.abs(rng.standard_normal(2000)) * 0.02])
    x = x[np.abs(x) < 65500.0]
    assert np.array_equal(orc.to_fp16(x), np.array([rational(v) for v in x]))


def test_effective_bits_in_paper_band():
    lo, hi = (float(v) for v in open(os.path.join(GOLDEN, "effective_bits.txt")).read().split("\n")[-2].split())
    b = orc.effective_weight_bits(11008, 4096, 64, 64, 32)
    assert lo <= b <= hi
    # independent count of the same storage in bytes
    bytes_ = 11008 * 4096 / 8 + 2 * 11008 + 2 * 32 * (4096 + 11008) + 4 * 2 * 64 * 64
    assert math.isclose(b, 8 * bytes_ / (11008 * 4096), rel_tol=1e-12)


# ------------------------------------------------------------------ input generator (storage grids only)
def test_inputs_are_on_their_storage_grids():
    import torch
    d = syn.make_layer(syn.CONFIGS["cfg0_tiny"])
    assert d.X.dtype == np.float32 and d.X.shape == (16, 512)
    cfg = syn.LayerConfig("t", 4, 64, 8, 8, 16, 4, "bf16", 2, 20.0, seed=1)
    e = syn.make_layer(cfg)
    xt = torch.from_numpy(e.X)
    assert torch.equal(xt.to(torch.bfloat16).to(torch.float32), xt)
    raw = np.random.default_rng(0).standard_normal(1000).astype(np.float32)
    assert torch.equal(torch.from_numpy(syn.round_to_bf16(raw)),
                       torch.from_numpy(raw).to(torch.bfloat16).to(torch.float32))
    assert np.array_equal(e.U.astype(np.float16).astype(np.float32), e.U)
    assert np.array_equal(e.V.astype(np.float16).astype(np.float32), e.V)
    # seeded: same config twice gives the same tensors
    f = syn.make_layer(cfg)
    assert np.array_equal(e.X, f.X) and np.array_equal(e.W, f.W)
    assert len(e.outlier_idx) == 2


def test_nibble_packing_layout_by_hand_and_round_trip():
    """Two 4-bit codes per byte: byte b of a run of 32 codes = code b (low nibble), code 16 + b (high
    nibble), two's complement -- written out for one run by hand, then the inverse on random codes."""
    q = np.zeros((1, 32), dtype=np.int64)
    q[0, 0], q[0, 16] = 1, 2          # byte 0 = 0x21
    q[0, 1], q[0, 17] = -1, 7         # byte 1 = 0x7f
    q[0, 15], q[0, 31] = -8, -7       # byte 15 = 0x98
    p = orc.pack_nibbles(q)
    assert p.shape == (1, 16) and p.dtype == np.uint8
    assert p[0, 0] == 0x21 and p[0, 1] == 0x7F and p[0, 15] == 0x98 and not np.any(p[0, 2:15])
    rng = np.random.default_rng(5)
    q = rng.integers(-7, 8, size=(5, 96))
    p = orc.pack_nibbles(q)
    assert p.shape == (5, 48) and np.array_equal(orc.unpack_nibbles(p), q)
    # the second run starts at byte 16 and pairs codes 32.. with 48..
    assert p[2, 16] == ((q[2, 32] & 0xF) | ((q[2, 48] & 0xF) << 4))
    for bad in (np.full((1, 32), 8), np.zeros((1, 48), dtype=np.int64)):
        with pytest.raises(ValueError):
            orc.pack_nibbles(bad)
