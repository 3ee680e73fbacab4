"""ctypes binding of the offline quantizer's C ABI (include/bwla_quantizer.h): the same names without
the `bwla_` prefix, argument marshalling only.  Tensors are torch CUDA tensors (fp64 for the step
calls); every computation runs in the library's HIP kernels."""
from __future__ import annotations

from ctypes import POINTER, byref, c_double, c_int32, c_int64, c_size_t, c_void_p

from . import binding as _b

EXPORTS = ["bwla_quantizer_workspace_size", "bwla_q_okt_rows", "bwla_q_init_theta", "bwla_q_em_step", "bwla_q_gmm_nll",
           "bwla_q_procrustes", "bwla_q_svd_square", "bwla_q_truncate_rank", "bwla_q_psp_step", "bwla_quantize_layer"]

_ready = False


def load():
    global _ready
    lib = _b.load()
    if _ready:
        return lib
    P, I64, I32, D, SZ = c_void_p, c_int64, c_int32, c_double, c_size_t
    lib.bwla_quantizer_workspace_size.argtypes = [I64, I64, I32, I32, I32, POINTER(c_size_t)]
    lib.bwla_q_okt_rows.argtypes = [P, P, P, I32, P, P, I64, I64, I32, I32, P, P, P, SZ, P]
    lib.bwla_q_init_theta.argtypes = [P, I64, I64, D, P, P, P]
    lib.bwla_q_em_step.argtypes = [P, I64, I64, D, P, P, P]
    lib.bwla_q_gmm_nll.argtypes = [P, I64, I64, P, P, P, P, SZ, P]
    lib.bwla_q_procrustes.argtypes = [I32, P, P, P, P, P, I64, I64, I32, I32, P, P, SZ, P]
    lib.bwla_q_svd_square.argtypes = [P, I32, P, P, P, P, SZ, P]
    lib.bwla_q_truncate_rank.argtypes = [P, I64, I64, I32, I32, D, P, P, P, P, SZ, P]
    lib.bwla_q_psp_step.argtypes = [P, P, P, I32, P, P, P, P, I64, I64, I32, I32, D, I32, D, P, SZ, P]
    lib.bwla_quantize_layer.argtypes = [P, I64, I64, I32, I32, I32, I32, D, D, I32, D, I32, P, P, P, P, P, P, P, P, P,
                                        SZ, P]
    for name in EXPORTS:
        getattr(lib, name).restype = c_int32
    _ready = True
    return lib


_p, _s, _ck = _b._ptr, _b._stream, _b._check


def workspace_size(n: int, m: int, n1: int, n2: int, k: int) -> int:
    out = c_size_t()
    _ck(load().bwla_quantizer_workspace_size(n, m, n1, n2, k, byref(out)), "bwla_quantizer_workspace_size")
    return out.value


def _ws(ws):
    return _p(ws), ws.numel() * ws.element_size()


def okt_rows(W, A, Bt, R1, R2, X, ybar, ws) -> None:
    n, m = W.shape
    k = 0 if A is None else A.shape[1]
    _ck(load().bwla_q_okt_rows(_p(W), _p(A), _p(Bt), k, _p(R1), _p(R2), n, m, R1.shape[0], R2.shape[0], _p(X),
                               _p(ybar), *_ws(ws), _s()), "bwla_q_okt_rows")


def init_theta(X, s2_min: float, c, s2) -> None:
    _ck(load().bwla_q_init_theta(_p(X), X.shape[0], X.shape[1], s2_min, _p(c), _p(s2), _s()), "bwla_q_init_theta")


def em_step(X, s2_min: float, c, s2) -> None:
    _ck(load().bwla_q_em_step(_p(X), X.shape[0], X.shape[1], s2_min, _p(c), _p(s2), _s()), "bwla_q_em_step")


def gmm_nll(X, c, s2, out, ws) -> None:
    _ck(load().bwla_q_gmm_nll(_p(X), X.shape[0], X.shape[1], _p(c), _p(s2), _p(out), *_ws(ws), _s()), "bwla_q_gmm_nll")


def procrustes(which: int, Wres, R1, R2, c, s2, Rnew, ws) -> None:
    n, m = Wres.shape
    _ck(load().bwla_q_procrustes(which, _p(Wres), _p(R1), _p(R2), _p(c), _p(s2), n, m, R1.shape[0], R2.shape[0],
                                 _p(Rnew), *_ws(ws), _s()), "bwla_q_procrustes")


def svd_square(G, sig, Ut, Vt, ws) -> None:
    _ck(load().bwla_q_svd_square(_p(G), G.shape[0], _p(sig), _p(Ut), _p(Vt), *_ws(ws), _s()), "bwla_q_svd_square")


def truncate_rank(Y, k: int, iters: int, tol: float, A, Bt, sig, ws) -> None:
    _ck(load().bwla_q_truncate_rank(_p(Y), Y.shape[0], Y.shape[1], k, iters, tol, _p(A), _p(Bt), _p(sig), *_ws(ws),
                                    _s()), "bwla_q_truncate_rank")


def psp_step(W, A, Bt, R1, R2, c, s2, mu: float, iters: int, tol: float, ws) -> None:
    n, m = W.shape
    _ck(load().bwla_q_psp_step(_p(W), _p(A), _p(Bt), A.shape[1], _p(R1), _p(R2), _p(c), _p(s2), n, m, R1.shape[0],
                               R2.shape[0], mu, iters, tol, *_ws(ws), _s()), "bwla_q_psp_step")


def quantize_layer(W, n1: int, n2: int, k: int, t_outer: int, R1, R2, W_rot, U, V, c, s2, hist, ws, mu: float = 0.0,
                   s2_min: float = 1e-8, svd_iters: int = 200, svd_tol: float = 1e-12,
                   init_identity: bool = True) -> None:
    n, m = W.shape
    _ck(load().bwla_quantize_layer(_p(W), n, m, n1, n2, k, t_outer, mu, s2_min, svd_iters, svd_tol,
                                   1 if init_identity else 0, _p(R1), _p(R2), _p(W_rot), _p(U), _p(V), _p(c), _p(s2),
                                   _p(hist), *_ws(ws), _s()), "bwla_quantize_layer")
