"""CPU oracle of the BWLA W1A6 quantized linear-layer forward.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, fp64 / exact-integer
NumPy implementation of what the HIP path computes.  Only the tests, the smoke check and
the benchmark's CPU-baseline leg may import it.  It shares no code with the HIP library and
imports nothing from the GPU package.

The method approximates Y = X W^T (it quantizes), so this oracle is the algorithm taken
step by step, not the dense product:

  1. rotate       X~ = X (R1 (x) R2)                       (paper Sec. 3.1, "OKT"; App. A.2.2,
                                                            "Matrix Formulation and Kronecker Structure")
  2. quantize     per-token symmetric INT6 of X~            (paper Sec. 4.1 "Implementation Details" names
                                                            per-token activation quantization; the symmetric
                                                            6-bit form [-31, 31] is this build's reading)
  3. binary GEMM  acc = q . Sign(W)^T  (exact integers)     (paper Sec. 3 "Discussion", Eq. 2-3)
  4. PSP branch   L = (X U) V^T                             (paper Sec. 3.2 "PSP": W_res = W - M, M = A B)
  5. dequantize   Y = s_t * alpha_n * acc + L               (paper Sec. 3 "Discussion", Eq. 4; App. A.2.4)

Variant with per-token asymmetric activation codes (paper Sec. 4.1 says "per-token asymmetric
quantization for activations", no formula): quantize_asym, forward_asym.

Variant with row-wise centering (paper Sec. 3 "Discussion", Eq. 1-2 and 4 in full): the shift
mu_n = mean_k W[n,k] is taken out before the sign and the scale are computed, and comes back at
dequantization: W_deq = delta_n Sign(W - mu_n) + mu_n, so Y = s_t (delta_n acc + mu_n qsum_t) + L
with qsum_t the sum of the token's codes (binarize_rows_centered, dequant_output_centered,
forward(..., centered=True)).

Block chaining: swiglu_interleaved is the gate between the merged gate|up projection and the down
projection of the MLP blocks the paper quantizes; to_bf16 the storage grid its result is kept on.

Pins (tests/test_oracle_pins.py, no GPU): every function below is checked against something
other than itself -- the dense Kronecker product, norm preservation and forward invariance,
hand-derived worked values, the closed-form optimal scale and its residual, brute-force loops,
and the exact end-to-end case.  The accuracy of the approximation itself (Y against the
unquantized X W^T on synthetic data) is *parity unpinned*: the paper only reports it through
perplexities of pretrained models.
"""
from __future__ import annotations

import math

import numpy as np

QMAX = 31  # symmetric INT6: codes in [-31, 31]; -32 is never produced


# --------------------------------------------------------------------------- Alg. 1
def kron_factor(n: int) -> tuple[int, int]:
    """Kronecker dimension factorization (paper App. A.1, Algorithm 1).

    Start at floor(sqrt(n)) and walk down to the closest divisor; that divisor is n2 and
    n1 = n / n2, so n1 >= n2.  A prime n gives (n, 1).
    """
    if n < 1:
        raise ValueError("n must be >= 1")
    a = math.isqrt(n)
    while a > 1 and n % a != 0:
        a -= 1
    n2 = a
    n1 = n // n2
    return n1, n2


# --------------------------------------------------------------------------- step 1
def kron_rotate(X: np.ndarray, R1: np.ndarray, R2: np.ndarray) -> np.ndarray:
    """X (M, K) times the Kronecker product R1 (x) R2, in fp64, without forming it.

    With the standard Kronecker product, (R1 (x) R2)[a*n2+b, c*n2+d] = R1[a,c] * R2[b,d].
    Reshaping a token row-major to V (n1, n2), the product is R1^T V R2 reshaped back
    (paper Sec. 3.1 OKT and App. A.2.2 write the same object with a column-major vec).
    """
    X = np.asarray(X, dtype=np.float64)
    R1 = np.asarray(R1, dtype=np.float64)
    R2 = np.asarray(R2, dtype=np.float64)
    n1, n2 = R1.shape[0], R2.shape[0]
    M, K = X.shape
    if R1.shape != (n1, n1) or R2.shape != (n2, n2) or n1 * n2 != K:
        raise ValueError("factor shapes do not match K")
    V = X.reshape(M, n1, n2)
    Z = np.matmul(V, R2)                 # Z[t,a,d] = sum_b V[t,a,b] R2[b,d]
    Y = np.matmul(R1.T, Z)               # Y[t,c,d] = sum_a R1[a,c] Z[t,a,d]
    return Y.reshape(M, K)


def kron_dense(R1: np.ndarray, R2: np.ndarray) -> np.ndarray:
    """The dense K x K rotation, entry by entry from the definition (small K only)."""
    R1 = np.asarray(R1, dtype=np.float64)
    R2 = np.asarray(R2, dtype=np.float64)
    n1, n2 = R1.shape[0], R2.shape[0]
    Q = np.empty((n1 * n2, n1 * n2), dtype=np.float64)
    for a in range(n1):
        for b in range(n2):
            for c in range(n1):
                Q[a * n2 + b, c * n2: (c + 1) * n2] = R1[a, c] * R2[b, :]
    return Q


# --------------------------------------------------------------------------- step 2
def quantize_sym(Xr: np.ndarray, bits: int = 6):
    """Per-token symmetric quantization to `bits` bits (this build's reading of paper Sec. 4.1;
    the paper evaluates 6- and 4-bit activations, Tables 1-3, and times W1A8, Sec. 4.4).

    With qmax = 2^(bits-1) - 1 (31 for INT6, 127 for INT8, 7 for INT4): amax_t = max_k |X~[t,k]|;
    v = qmax X~ / amax_t;  q = clip(rint(v), -qmax, qmax) with ties to even;  s_t = amax_t / qmax.
    A token that is all zero gets q = 0 and s = 0.
    Returns (q int8 (M,K), s fp64 (M,), v fp64 (M,K)); v is the pre-rounding value the parity
    test needs for its rounding-boundary mask.
    """
    if bits < 2 or bits > 8:
        raise ValueError("bits must be in 2..8 (codes are kept in int8)")
    qmax = (1 << (bits - 1)) - 1
    Xr = np.asarray(Xr, dtype=np.float64)
    amax = np.max(np.abs(Xr), axis=1)
    safe = np.where(amax > 0, amax, 1.0)
    v = Xr * (qmax / safe)[:, None]
    v[amax == 0] = 0.0
    q = np.clip(np.rint(v), -qmax, qmax).astype(np.int8)
    s = amax / qmax
    return q, s, v


def quantize_asym(Xr: np.ndarray, bits: int = 6):
    """Per-token asymmetric quantization (paper Sec. 4.1 names it, without a formula; this is the
    usual min-max affine form, this build's reading): with L = 2^bits - 1 levels above zero,
        lo_t = min(min_k X~[t,k], 0),  hi_t = max(max_k X~[t,k], 0)      (zero is representable)
        s_t = (hi_t - lo_t) / L,   z_t = rint(-lo_t / s_t)  in [0, L]     (the zero point)
        q = clip(rint(X~ / s_t) + z_t, 0, L),  dequantized value s_t (q - z_t);
    ties to even; an all-zero token gets q = z = 0 and s = 0.
    Returns (q int16 (M,K) in [0, L], s fp64 (M,), z int64 (M,), v fp64 (M,K) = X~ / s_t, the
    pre-rounding value, and u fp64 (M,) = -lo_t / s_t, the pre-rounding zero point)."""
    if bits < 2 or bits > 8:
        raise ValueError("bits must be in 2..8")
    L = (1 << bits) - 1
    Xr = np.asarray(Xr, dtype=np.float64)
    lo = np.minimum(Xr.min(axis=1), 0.0)
    hi = np.maximum(Xr.max(axis=1), 0.0)
    span = hi - lo
    s = span / L
    safe = np.where(span > 0, s, 1.0)
    u = np.where(span > 0, -lo / safe, 0.0)
    z = np.rint(u).astype(np.int64)
    v = Xr / safe[:, None]
    v[span == 0] = 0.0
    q = np.clip(np.rint(v) + z[:, None], 0, L).astype(np.int16)
    return q, s, z, v, u


def quantize_int6(Xr: np.ndarray):
    """Per-token symmetric INT6: quantize_sym with 6 bits (codes in [-31, 31])."""
    return quantize_sym(Xr, 6)


# --------------------------------------------------------------------------- step 3 (offline part)
def binarize_rows(W: np.ndarray):
    """Row-wise binarization without shift (paper Sec. 3 Eq. 2-3; App. A.2.4).

    Sign(x) = +1 for x > 0 and -1 for x <= 0 (Eq. 3).  The per-output-channel scale is the
    mean magnitude of the row, the minimizer of sum_j (w_j - alpha sign(w_j))^2 (App. A.2.4).
    Returns (sgn int8 (N,K) in {-1,+1}, alpha fp64 (N,)).
    """
    W = np.asarray(W, dtype=np.float64)
    sgn = np.where(W > 0, 1, -1).astype(np.int8)
    alpha = np.mean(np.abs(W), axis=1)
    return sgn, alpha


def binarize_rows_centered(W: np.ndarray):
    """Row-wise binarization with the shift (paper Sec. 3 "Discussion", Eq. 1-2):
    mu_n = mean_k W[n,k], delta_n = mean_k |W[n,k] - mu_n|, sign of the centered weight, with
    Sign(0) = -1 (Eq. 3).  Returns (sgn int8 (N,K) in {-1,+1}, delta fp64 (N,), mu fp64 (N,))."""
    W = np.asarray(W, dtype=np.float64)
    mu = np.mean(W, axis=1)
    C = W - mu[:, None]
    sgn = np.where(C > 0, 1, -1).astype(np.int8)
    delta = np.mean(np.abs(C), axis=1)
    return sgn, delta, mu


def to_fp16(a: np.ndarray) -> np.ndarray:
    """Round to the fp16 storage grid (nearest even) and return as fp64."""
    return np.asarray(a, dtype=np.float64).astype(np.float16).astype(np.float64)


# --------------------------------------------------------------------------- step 3 (online part)
def binary_gemm(q: np.ndarray, sgn: np.ndarray) -> np.ndarray:
    """acc[t,n] = sum_k q[t,k] * sgn[n,k], exact.

    |acc| <= 31 K is far below 2^53, so the fp64 matrix product of the integer-valued
    operands is exact in any summation order; it is returned as int64.
    """
    q = np.asarray(q)
    sgn = np.asarray(sgn)
    acc = np.matmul(q.astype(np.float64), sgn.astype(np.float64).T)
    return np.rint(acc).astype(np.int64)


def binary_gemm_loops(q, sgn):
    """The same contraction as a literal triple loop over Python ints (tiny sizes only)."""
    M, K = len(q), len(q[0])
    N = len(sgn)
    out = [[0] * N for _ in range(M)]
    for t in range(M):
        for n in range(N):
            a = 0
            for k in range(K):
                a += int(q[t][k]) * int(sgn[n][k])
            out[t][n] = a
    return np.array(out, dtype=np.int64)


# --------------------------------------------------------------------------- step 4
def psp_project(X: np.ndarray, U: np.ndarray) -> np.ndarray:
    """T = X U (M, r): the low-rank branch reads the original, un-rotated, un-quantized input
    (paper Sec. 3.2: the residual M = A B lives in the un-rotated coordinates)."""
    return np.asarray(X, dtype=np.float64) @ np.asarray(U, dtype=np.float64)


# --------------------------------------------------------------------------- step 5
def dequant_output(acc, s, alpha, T=None, V=None) -> np.ndarray:
    """Y[t,n] = s_t * alpha_n * acc[t,n] + sum_j T[t,j] V[n,j]   (paper Eq. 4 without shift;
    Sec. 3.2 for the added low-rank term)."""
    Y = np.asarray(s, dtype=np.float64)[:, None] * np.asarray(alpha, dtype=np.float64)[None, :] \
        * np.asarray(acc, dtype=np.float64)
    if T is not None and V is not None and np.asarray(T).shape[1] > 0:
        Y = Y + np.asarray(T, dtype=np.float64) @ np.asarray(V, dtype=np.float64).T
    return Y


def dequant_output_centered(acc, s, delta, mu, qsum, T=None, V=None) -> np.ndarray:
    """Dequantization with the shift (paper Sec. 3 "Discussion", Eq. 4: W_deq = W~ delta + mu):
    the dequantized token s_t q[t,:] times W_deq[n,:] = delta_n sgn[n,:] + mu_n gives
    Y[t,n] = s_t * (delta_n * acc[t,n] + mu_n * qsum_t) + sum_j T[t,j] V[n,j],  qsum_t = sum_k q[t,k]."""
    s = np.asarray(s, dtype=np.float64)[:, None]
    Y = s * (np.asarray(delta, dtype=np.float64)[None, :] * np.asarray(acc, dtype=np.float64)
             + np.asarray(mu, dtype=np.float64)[None, :] * np.asarray(qsum, dtype=np.float64)[:, None])
    if T is not None and V is not None and np.asarray(T).shape[1] > 0:
        Y = Y + np.asarray(T, dtype=np.float64) @ np.asarray(V, dtype=np.float64).T
    return Y


# --------------------------------------------------------------------------- whole path
def forward_asym(X, R1, R2, W_rot, U=None, V=None, centered: bool = False, act_bits: int = 6) -> dict:
    """The path with per-token asymmetric activation codes (quantize_asym): the dequantized token
    s_t (q - z_t) meets the dequantized weights, alpha_n sgn (+ mu_n with centered=True):
        Y[t,n] = s_t * (alpha_n * sum_k (q[t,k] - z_t) sgn[n,k] + mu_n * sum_k (q[t,k] - z_t)) + L[t,n].
    The contraction runs on the centered codes q - z, exact integers."""
    Xr = kron_rotate(X, R1, R2)
    q, s, z, v, u = quantize_asym(Xr, act_bits)
    c = q.astype(np.int64) - z[:, None]                   # centered codes, |c| <= 2^bits - 1
    if centered:
        sgn, alpha, mu = binarize_rows_centered(W_rot)
        mu16 = to_fp16(mu)
    else:
        sgn, alpha = binarize_rows(W_rot)
        mu = None
        mu16 = np.zeros(np.asarray(W_rot).shape[0])
    alpha16 = to_fp16(alpha)
    acc_c = c.astype(np.float64) @ sgn.astype(np.float64).T   # exact: |acc| <= 255 K < 2^53
    acc_c = np.rint(acc_c).astype(np.int64)
    if U is not None and np.asarray(U).size > 0:
        T = psp_project(X, U)
    else:
        T = np.zeros((np.asarray(X).shape[0], 0))
        V = np.zeros((np.asarray(W_rot).shape[0], 0))
    Y = dequant_output_centered(acc_c, s, alpha16, mu16, c.sum(axis=1), T, V)
    return dict(Xr=Xr, q=q, s=s, z=z, v=v, u=u, c=c, sgn=sgn, alpha=alpha, alpha16=alpha16, mu=mu,
                acc_c=acc_c, T=T, Y=Y)


def forward(X, R1, R2, W_rot, U=None, V=None, centered: bool = False, act_bits: int = 6) -> dict:
    """The whole hot path on stored parameter values.

    X      (M,K)  activations as stored (already on the bf16 or fp32 grid)
    R1,R2  fp32 orthogonal factors
    W_rot  (N,K)  the weight matrix in rotated (and PSP-corrected) coordinates, fp32
    U (K,r), V (N,r): PSP factors on the fp16 grid, or None / r = 0
    The scale alpha (and, with centered=True, the shift mu) is rounded to fp16 because that is
    how the layer stores it.  centered=True: binarization with the row shift (Eq. 1-2, 4).
    """
    Xr = kron_rotate(X, R1, R2)
    q, s, v = quantize_sym(Xr, act_bits)
    qsum = q.astype(np.int64).sum(axis=1)
    if centered:
        sgn, alpha, mu = binarize_rows_centered(W_rot)
        mu16 = to_fp16(mu)
    else:
        sgn, alpha = binarize_rows(W_rot)
        mu = mu16 = None
    alpha16 = to_fp16(alpha)
    acc = binary_gemm(q, sgn)
    if U is not None and np.asarray(U).size > 0:
        T = psp_project(X, U)
    else:
        T = np.zeros((np.asarray(X).shape[0], 0))
        V = np.zeros((np.asarray(W_rot).shape[0], 0))
    if centered:
        Y = dequant_output_centered(acc, s, alpha16, mu16, qsum, T, V)
    else:
        Y = dequant_output(acc, s, alpha16, T, V)
    return dict(Xr=Xr, q=q, s=s, v=v, sgn=sgn, alpha=alpha, alpha16=alpha16, mu=mu, mu16=mu16,
                acc=acc, T=T, Y=Y, qsum=qsum)


def forward_rows(X, R1, R2, sgn, alpha16, U, V, rows, mu16=None, act_bits: int = 6) -> dict:
    """The path for a subset of token rows (tokens are independent: per-token scale,
    row-wise products).  Used where the full M would take minutes on the CPU.  With mu16 the
    layer is one with row shifts (sgn, alpha16 from binarize_rows_centered)."""
    Xs = np.asarray(X)[rows]
    Xr = kron_rotate(Xs, R1, R2)
    q, s, v = quantize_sym(Xr, act_bits)
    acc = binary_gemm(q, sgn)
    if U is not None and np.asarray(U).size > 0:
        T = psp_project(Xs, U)
    else:
        T = np.zeros((Xs.shape[0], 0))
        V = np.zeros((np.asarray(sgn).shape[0], 0))
    qsum = q.astype(np.int64).sum(axis=1)
    if mu16 is not None:
        Y = dequant_output_centered(acc, s, alpha16, mu16, qsum, T, V)
    else:
        Y = dequant_output(acc, s, alpha16, T, V)
    return dict(Xr=Xr, q=q, s=s, v=v, acc=acc, T=T, Y=Y, qsum=qsum)


def forward_loops(X, R1, R2, W_rot, U, V) -> np.ndarray:
    """Everything as scalar Python loops on the dense definition (tiny sizes only):
    dense Kronecker matrix, per-token max, round-half-even, sign, mean magnitude, sums."""
    X = [[float(x) for x in row] for row in np.asarray(X, dtype=np.float64)]
    Q = kron_dense(R1, R2).tolist()
    W = np.asarray(W_rot, dtype=np.float64).tolist()
    U = np.asarray(U, dtype=np.float64).tolist() if U is not None else []
    V = np.asarray(V, dtype=np.float64).tolist() if V is not None else []
    M, K, N = len(X), len(X[0]), len(W)
    r = len(U[0]) if U else 0
    Y = np.zeros((M, N))
    for t in range(M):
        xr = [math.fsum(X[t][i] * Q[i][k] for i in range(K)) for k in range(K)]
        amax = max(abs(z) for z in xr)
        qs = [0] * K
        if amax > 0:
            for k in range(K):
                c = round(31.0 * xr[k] / amax)       # Python's round is half-to-even
                qs[k] = max(-31, min(31, c))
        st = amax / 31.0
        Tt = [math.fsum(X[t][k] * U[k][j] for k in range(K)) for j in range(r)]
        for n in range(N):
            alpha = float(np.float16(math.fsum(abs(w) for w in W[n]) / K))
            acc = 0
            for k in range(K):
                acc += qs[k] if W[n][k] > 0 else -qs[k]
            low = math.fsum(Tt[j] * V[n][j] for j in range(r))
            Y[t, n] = st * alpha * acc + low
    return Y


# --------------------------------------------------------------------------- accounting
# --------------------------------------------------------------------------- gated MLP (block chaining)
def to_bf16(a: np.ndarray) -> np.ndarray:
    """Round to the bfloat16 grid (nearest, ties to even) and return as fp64.  bfloat16 is the
    upper half of an fp32 word: round the fp64 value to fp32 first only where that is exact
    enough -- here the rounding is done on the fp64 value directly, by scaling to the 8-bit
    significand, so that no double rounding can occur."""
    a = np.asarray(a, dtype=np.float64)
    out = np.zeros_like(a)
    nz = (a != 0) & np.isfinite(a)
    m, e = np.frexp(a[nz])                     # a = m * 2^e, 0.5 <= |m| < 1
    out[nz] = np.ldexp(np.rint(m * 256.0), e - 8)   # 8 significant bits; np.rint rounds ties to even
    out[~np.isfinite(a)] = a[~np.isfinite(a)]
    return out


def swiglu_interleaved(Y: np.ndarray) -> np.ndarray:
    """The gate of the MLP blocks of the models the paper quantizes (their up, gate and down
    projections: paper App., loss trajectories of the MLP blocks): h = silu(g) * u with
    silu(g) = g / (1 + exp(-g)).  The nonlinearity is the model's, not the paper's method.
    Y holds the outputs of a layer whose rows interleave the two projections: column 2 i is
    gate channel i, column 2 i + 1 is up channel i.  Returns h (fp64, not rounded), [M, N / 2]."""
    Y = np.asarray(Y, dtype=np.float64)
    g, u = Y[:, 0::2], Y[:, 1::2]
    with np.errstate(over="ignore"):
        return g / (1.0 + np.exp(-g)) * u


def pack_nibbles(q: np.ndarray) -> np.ndarray:
    """4-bit codes two to a byte (paper Table 3, W1A4; the storage layout is this build's): K is cut
    into runs of 32 codes, and byte b (0..15) of run j holds code 32 j + b in its low nibble and code
    32 j + 16 + b in its high nibble, both in two's complement.  q: (M, K) integers in [-8, 7]."""
    q = np.asarray(q, dtype=np.int64)
    M, K = q.shape
    if K % 32 != 0 or q.min() < -8 or q.max() > 7:
        raise ValueError("need K % 32 == 0 and codes in [-8, 7]")
    runs = q.reshape(M, K // 32, 2, 16)
    return ((runs[:, :, 0, :] & 0xF) | ((runs[:, :, 1, :] & 0xF) << 4)).reshape(M, K // 2).astype(np.uint8)


def unpack_nibbles(p: np.ndarray) -> np.ndarray:
    """Inverse of pack_nibbles: (M, K / 2) bytes -> (M, K) codes."""
    p = np.asarray(p, dtype=np.int64)
    M, KB = p.shape
    runs = p.reshape(M, KB // 16, 16)
    sext = lambda n: np.where(n >= 8, n - 16, n)
    out = np.stack([sext(runs & 0xF), sext((runs >> 4) & 0xF)], axis=2)
    return out.reshape(M, 2 * KB)


def effective_weight_bits(N: int, K: int, n1: int, n2: int, r: int) -> float:
    """Stored bits per weight of one packed layer: 1 sign bit, fp16 scale per row, fp16 PSP
    factors U (K,r) and V (N,r), fp32 Kronecker factors (paper Table 1 reports 1.15-1.19)."""
    return 1.0 + (16.0 * (r * (K + N) + N) + 32.0 * (n1 * n1 + n2 * n2)) / (N * K)
