"""ctypes binding of libbwla: same names as the C ABI in include/bwla.h, argument marshalling
only.  Device memory and streams come from PyTorch; every step of the path runs in the HIP
kernels of the library.  There is no fallback: if the library is missing, loading raises."""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, byref, c_char_p, c_int, c_int32, c_int64, c_size_t, c_uint64, c_void_p

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libbwla.so")

BWLA_OK = 0
BWLA_ERR_NULL, BWLA_ERR_SHAPE, BWLA_ERR_ALIGN, BWLA_ERR_BUFSIZE, BWLA_ERR_UNSUPPORTED, BWLA_ERR_HIP = 1, 2, 3, 4, 5, 6
BWLA_X_F32, BWLA_X_BF16 = 0, 1
BWLA_MODE_ROW_SHIFT, BWLA_MODE_ASYM_ACT = 1, 2

EXPORTS = ["bwla_status_string", "bwla_version", "bwla_kron_factor", "bwla_packed_size", "bwla_pack_weights",
           "bwla_unpack_signs", "bwla_psp_workspace_size", "bwla_rotate_quant", "bwla_code_sums",
           "bwla_linear_forward", "bwla_decode_forward", "bwla_packed_size_centered", "bwla_pack_weights_centered", "bwla_rotate_quant_bits",
           "bwla_packed_size_mode", "bwla_pack_weights_mode", "bwla_swiglu_workspace_size",
           "bwla_linear_forward_swiglu", "bwla_decode_forward_static", "bwla_probe_hbm_read",
           "bwla_probe_mfma_int8", "bwla_decode_forward_launches", "bwla_decode_forward_bits", "bwla_pack_codes_a4",
           "bwla_linear_forward_a4", "bwla_probe_empty_launch", "bwla_probe_load_latency", "bwla_probe_clock"]


class BwlaLayer(Structure):
    _fields_ = [("N", c_int64), ("K", c_int64), ("n1", c_int32), ("n2", c_int32), ("r", c_int32),
                ("mode", c_int32), ("off_bits", c_uint64), ("off_alpha", c_uint64), ("off_V", c_uint64),
                ("off_U", c_uint64), ("off_R1", c_uint64), ("off_R2", c_uint64), ("off_R1p", c_uint64), ("off_R2p", c_uint64),
                ("off_Rd", c_uint64), ("blob_bytes", c_uint64),
                ("d_blob", c_void_p)]


class BwlaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def load() -> ctypes.CDLL:
    """Load libbwla.so from the package directory (build it first with build.py)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_2605_00422_amd.build` "
                                "(or __graft_entry__.build()) first")
    lib = ctypes.CDLL(LIB_PATH)
    lib.bwla_status_string.restype = c_char_p
    lib.bwla_status_string.argtypes = [c_int]
    lib.bwla_version.restype = c_int
    lib.bwla_kron_factor.argtypes = [c_int64, POINTER(c_int32), POINTER(c_int32)]
    lib.bwla_packed_size.argtypes = [c_int64, c_int64, c_int32, c_int32, c_int32, POINTER(c_size_t)]
    lib.bwla_pack_weights.argtypes = [c_void_p] * 5 + [c_int64, c_int64, c_int32, c_int32, c_int32, c_void_p,
                                                       c_size_t, c_void_p, POINTER(BwlaLayer)]
    lib.bwla_packed_size_centered.argtypes = lib.bwla_packed_size.argtypes
    lib.bwla_pack_weights_centered.argtypes = lib.bwla_pack_weights.argtypes
    lib.bwla_packed_size_mode.argtypes = [c_int64, c_int64, c_int32, c_int32, c_int32, c_int32, POINTER(c_size_t)]
    lib.bwla_pack_weights_mode.argtypes = [c_void_p] * 5 + [c_int64, c_int64, c_int32, c_int32, c_int32, c_int32,
                                                            c_void_p, c_size_t, c_void_p, POINTER(BwlaLayer)]
    lib.bwla_unpack_signs.argtypes = [POINTER(BwlaLayer), c_void_p, c_void_p, c_void_p]
    lib.bwla_psp_workspace_size.argtypes = [POINTER(BwlaLayer), c_int64, POINTER(c_size_t)]
    lib.bwla_rotate_quant.argtypes = [POINTER(BwlaLayer), c_void_p, c_int, c_int64, c_void_p, c_void_p, c_void_p,
                                      c_void_p, c_void_p, c_size_t, c_void_p]
    lib.bwla_rotate_quant_bits.argtypes = [POINTER(BwlaLayer), c_void_p, c_int, c_int, c_int64, c_void_p, c_void_p,
                                           c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
    lib.bwla_code_sums.argtypes = [c_void_p, c_int64, c_int64, c_void_p, c_void_p]
    lib.bwla_linear_forward.argtypes = [POINTER(BwlaLayer), c_void_p, c_void_p, c_void_p, c_void_p, c_int64,
                                        c_void_p, c_void_p, c_void_p]
    lib.bwla_decode_forward.argtypes = [POINTER(BwlaLayer), c_void_p, c_int, c_int64, c_void_p, c_void_p, c_void_p,
                                        c_void_p, c_void_p, c_size_t, c_void_p, c_void_p, c_void_p]
    lib.bwla_decode_forward_static.argtypes = [POINTER(BwlaLayer), c_void_p, c_int, c_int64, c_void_p, c_void_p,
                                               c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.bwla_decode_forward_bits.argtypes = [POINTER(BwlaLayer), c_void_p, c_int, c_int, c_int64, c_void_p, c_void_p, c_void_p,
                                             c_void_p, c_void_p, c_size_t, c_void_p, c_void_p, c_void_p]
    lib.bwla_pack_codes_a4.argtypes = [c_void_p, c_int64, c_int64, c_void_p, c_void_p]
    lib.bwla_linear_forward_a4.argtypes = [POINTER(BwlaLayer), c_void_p, c_void_p, c_void_p, c_void_p, c_int64,
                                           c_void_p, c_void_p, c_void_p]
    lib.bwla_decode_forward_launches.argtypes = [POINTER(BwlaLayer), c_int, c_int64, POINTER(c_int)]
    lib.bwla_probe_hbm_read.argtypes = [c_void_p, c_size_t, c_void_p, c_size_t, c_void_p]
    lib.bwla_probe_mfma_int8.argtypes = [c_int, c_void_p, c_size_t, POINTER(ctypes.c_int64), c_void_p]
    lib.bwla_probe_empty_launch.argtypes = [c_void_p]
    lib.bwla_probe_clock.argtypes = [c_void_p, c_void_p]
    lib.bwla_probe_load_latency.argtypes = [c_void_p, c_size_t, c_size_t, c_int, c_void_p, c_void_p]
    lib.bwla_swiglu_workspace_size.argtypes = [POINTER(BwlaLayer), c_int64, POINTER(c_size_t)]
    lib.bwla_linear_forward_swiglu.argtypes = [POINTER(BwlaLayer), c_void_p, c_void_p, c_void_p, c_void_p, c_int64,
                                               c_void_p, c_void_p, c_size_t, c_void_p]
    for name in EXPORTS:
        if name not in ("bwla_status_string", "bwla_version"):
            getattr(lib, name).restype = c_int
    _lib = lib
    return lib


def _check(status: int, where: str) -> None:
    if status != BWLA_OK:
        raise BwlaError(status, where)


def _ptr(t):
    return None if t is None else c_void_p(t.data_ptr())


def _stream():
    import torch
    return c_void_p(torch.cuda.current_stream().cuda_stream)


# ------------------------------------------------------------------ host-only calls
def status_string(status: int) -> str:
    return load().bwla_status_string(int(status)).decode()


def version() -> int:
    return load().bwla_version()


def kron_factor(K: int) -> tuple[int, int]:
    n1, n2 = c_int32(), c_int32()
    _check(load().bwla_kron_factor(K, byref(n1), byref(n2)), "bwla_kron_factor")
    return n1.value, n2.value


def packed_size(N: int, K: int, n1: int, n2: int, r: int, centered: bool = False, asym: bool = False) -> int:
    out = c_size_t()
    if asym:
        mode = BWLA_MODE_ASYM_ACT | (BWLA_MODE_ROW_SHIFT if centered else 0)
        _check(load().bwla_packed_size_mode(N, K, n1, n2, r, mode, byref(out)), "bwla_packed_size_mode")
        return out.value
    name = "bwla_packed_size_centered" if centered else "bwla_packed_size"
    _check(getattr(load(), name)(N, K, n1, n2, r, byref(out)), name)
    return out.value


# ------------------------------------------------------------------ device calls (torch tensors in, torch tensors out)
class PackedLayer:
    """Owns the device blob (a torch uint8 tensor) and the plain descriptor."""

    def __init__(self, desc: BwlaLayer, blob):
        self.desc = desc
        self.blob = blob

    @property
    def shape(self):
        d = self.desc
        return d.N, d.K, d.n1, d.n2, d.r


def pack_weights(W_rot, R1, R2, U, V, n1: int, n2: int, centered: bool = False, asym: bool = False) -> PackedLayer:
    """W_rot (N,K), R1, R2, U (K,r), V (N,r): fp32 CUDA tensors (U, V may be None for r = 0).
    centered: binarize with the row shift (bwla_pack_weights_centered); asym: the layer's
    activations get per-token asymmetric codes (bwla_pack_weights_mode)."""
    import torch
    N, K = W_rot.shape
    r = 0 if U is None else U.shape[1]
    nbytes = packed_size(N, K, n1, n2, r, centered, asym)
    blob = torch.zeros(nbytes, dtype=torch.uint8, device=W_rot.device)
    desc = BwlaLayer()
    if asym:
        mode = BWLA_MODE_ASYM_ACT | (BWLA_MODE_ROW_SHIFT if centered else 0)
        _check(load().bwla_pack_weights_mode(_ptr(W_rot), _ptr(R1), _ptr(R2), _ptr(U), _ptr(V), N, K, n1, n2, r, mode,
                                             _ptr(blob), nbytes, _stream(), byref(desc)), "bwla_pack_weights_mode")
        return PackedLayer(desc, blob)
    name = "bwla_pack_weights_centered" if centered else "bwla_pack_weights"
    _check(getattr(load(), name)(_ptr(W_rot), _ptr(R1), _ptr(R2), _ptr(U), _ptr(V), N, K, n1, n2, r,
                                 _ptr(blob), nbytes, _stream(), byref(desc)), name)
    return PackedLayer(desc, blob)


def unpack_signs(layer: PackedLayer):
    import torch
    N, K = layer.desc.N, layer.desc.K
    sgn = torch.empty((N, K), dtype=torch.int8, device=layer.blob.device)
    alpha = torch.empty((N,), dtype=torch.float32, device=layer.blob.device)
    _check(load().bwla_unpack_signs(byref(layer.desc), _ptr(sgn), _ptr(alpha), _stream()), "bwla_unpack_signs")
    return sgn, alpha


def psp_workspace_size(layer: PackedLayer, M: int) -> int:
    out = c_size_t()
    _check(load().bwla_psp_workspace_size(byref(layer.desc), M, byref(out)), "bwla_psp_workspace_size")
    return out.value


class Activations:
    """Caller-owned outputs of bwla_rotate_quant for M tokens (allocated once, reused)."""

    def __init__(self, layer: PackedLayer, M: int):
        import torch
        dev = layer.blob.device
        d = layer.desc
        self.M = M
        self.q = torch.empty((M, d.K), dtype=torch.int8, device=dev)
        self.scale = torch.empty((M,), dtype=torch.float32, device=dev)
        self.qsum = torch.empty((M,), dtype=torch.int32, device=dev)
        self.T = torch.empty((M, d.r), dtype=torch.float32, device=dev) if d.r > 0 else None
        ws = psp_workspace_size(layer, M)
        self.ws_bytes = ws
        self.ws = torch.zeros(max(ws, 16), dtype=torch.uint8, device=dev)   # zero-filled once, as the ABI asks


def rotate_quant(layer: PackedLayer, X, act: Activations, act_bits: int = 6) -> Activations:
    """X: (M,K) CUDA tensor, float32 or bfloat16.  act_bits other than 6: bwla_rotate_quant_bits."""
    import torch
    xd = BWLA_X_BF16 if X.dtype == torch.bfloat16 else BWLA_X_F32
    if X.dtype not in (torch.bfloat16, torch.float32):
        raise TypeError("X must be float32 or bfloat16")
    if act_bits == 6:
        _check(load().bwla_rotate_quant(byref(layer.desc), _ptr(X), xd, X.shape[0], _ptr(act.q), _ptr(act.scale),
                                        _ptr(act.qsum), _ptr(act.T), _ptr(act.ws), act.ws_bytes, _stream()),
               "bwla_rotate_quant")
    else:
        _check(load().bwla_rotate_quant_bits(byref(layer.desc), _ptr(X), xd, act_bits, X.shape[0], _ptr(act.q),
                                             _ptr(act.scale), _ptr(act.qsum), _ptr(act.T), _ptr(act.ws),
                                             act.ws_bytes, _stream()), "bwla_rotate_quant_bits")
    return act


def decode_forward(layer: PackedLayer, X, act: Activations, Y, acc=None, act_bits: int = 6):
    """bwla_rotate_quant + bwla_linear_forward in one call (one kernel launch where possible)."""
    import torch
    if X.dtype not in (torch.bfloat16, torch.float32):
        raise TypeError("X must be float32 or bfloat16")
    xd = BWLA_X_BF16 if X.dtype == torch.bfloat16 else BWLA_X_F32
    if act_bits == 6:
        _check(load().bwla_decode_forward(byref(layer.desc), _ptr(X), xd, X.shape[0], _ptr(act.q), _ptr(act.scale),
                                          _ptr(act.qsum), _ptr(act.T), _ptr(act.ws), act.ws_bytes, _ptr(Y), _ptr(acc),
                                          _stream()), "bwla_decode_forward")
    else:
        _check(load().bwla_decode_forward_bits(byref(layer.desc), _ptr(X), xd, int(act_bits), X.shape[0], _ptr(act.q),
                                               _ptr(act.scale), _ptr(act.qsum), _ptr(act.T), _ptr(act.ws), act.ws_bytes,
                                               _ptr(Y), _ptr(acc), _stream()), "bwla_decode_forward_bits")
    return Y


def decode_forward_launches(layer: PackedLayer, M: int, bf16: bool = True) -> int:
    n = c_int()
    _check(load().bwla_decode_forward_launches(byref(layer.desc), BWLA_X_BF16 if bf16 else BWLA_X_F32, M, byref(n)),
           "bwla_decode_forward_launches")
    return n.value


def decode_forward_static(layer: PackedLayer, X, act: Activations, Y, acc=None):
    """bwla_decode_forward with the library's own fixed scratch (act.ws is not used)."""
    import torch
    if X.dtype not in (torch.bfloat16, torch.float32):
        raise TypeError("X must be float32 or bfloat16")
    xd = BWLA_X_BF16 if X.dtype == torch.bfloat16 else BWLA_X_F32
    _check(load().bwla_decode_forward_static(byref(layer.desc), _ptr(X), xd, X.shape[0], _ptr(act.q), _ptr(act.scale),
                                             _ptr(act.qsum), _ptr(act.T), _ptr(Y), _ptr(acc), _stream()),
           "bwla_decode_forward_static")
    return Y


def probe_hbm_read(src, sink) -> None:
    """One streaming read of the whole tensor `src` (measurement aid)."""
    _check(load().bwla_probe_hbm_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink),
                                      sink.numel() * sink.element_size(), _stream()), "bwla_probe_hbm_read")


def probe_mfma_int8(iters: int, sink) -> int:
    """One launch of back-to-back INT8 MFMAs (measurement aid); returns its operation count."""
    ops = ctypes.c_int64()
    _check(load().bwla_probe_mfma_int8(int(iters), _ptr(sink), sink.numel() * sink.element_size(), byref(ops),
                                       _stream()), "bwla_probe_mfma_int8")
    return ops.value


def probe_empty_launch() -> None:
    _check(load().bwla_probe_empty_launch(_stream()), "bwla_probe_empty_launch")


def probe_clock(out) -> None:
    """out: int64 CUDA tensor of one element; gets the GPU's 100 MHz counter when the launch runs."""
    _check(load().bwla_probe_clock(_ptr(out), _stream()), "bwla_probe_clock")


def probe_load_latency(buf, stride_bytes: int, iters: int, out) -> None:
    """out: int64 CUDA tensor of two elements (ticks of 10 ns, last index)."""
    _check(load().bwla_probe_load_latency(_ptr(buf), buf.numel() * buf.element_size(), stride_bytes, iters, _ptr(out),
                                          _stream()), "bwla_probe_load_latency")


def pack_codes_a4(q, q4=None):
    """int8 codes in [-8, 7] (M x K) -> nibble-packed codes (M x K / 2 bytes)."""
    import torch
    if q4 is None:
        q4 = torch.empty((q.shape[0], q.shape[1] // 2), dtype=torch.uint8, device=q.device)
    _check(load().bwla_pack_codes_a4(_ptr(q), q.shape[0], q.shape[1], _ptr(q4), _stream()), "bwla_pack_codes_a4")
    return q4


def linear_forward_a4(layer: PackedLayer, q4, act: Activations, Y, acc=None):
    """bwla_linear_forward on nibble-packed 4-bit codes (scale, code sums and T from `act`)."""
    _check(load().bwla_linear_forward_a4(byref(layer.desc), _ptr(q4), _ptr(act.scale), _ptr(act.qsum), _ptr(act.T),
                                         act.M, _ptr(Y), _ptr(acc), _stream()), "bwla_linear_forward_a4")
    return Y


def code_sums(q, qsum) -> None:
    _check(load().bwla_code_sums(_ptr(q), q.shape[0], q.shape[1], _ptr(qsum), _stream()), "bwla_code_sums")


def swiglu_workspace_size(layer: PackedLayer, M: int) -> int:
    out = c_size_t()
    _check(load().bwla_swiglu_workspace_size(byref(layer.desc), M, byref(out)), "bwla_swiglu_workspace_size")
    return out.value


def linear_forward_swiglu(layer: PackedLayer, act: Activations, H, ws=None):
    """H (bf16, M x N/2) = silu(gate) * up of a layer whose rows interleave gate and up channels."""
    nbytes = 0 if ws is None else ws.numel() * ws.element_size()
    _check(load().bwla_linear_forward_swiglu(byref(layer.desc), _ptr(act.q), _ptr(act.scale), _ptr(act.qsum),
                                             _ptr(act.T), act.M, _ptr(H), _ptr(ws), nbytes, _stream()),
           "bwla_linear_forward_swiglu")
    return H


def linear_forward(layer: PackedLayer, act: Activations, Y, acc=None):
    _check(load().bwla_linear_forward(byref(layer.desc), _ptr(act.q), _ptr(act.scale), _ptr(act.qsum), _ptr(act.T),
                                      act.M, _ptr(Y), _ptr(acc), _stream()), "bwla_linear_forward")
    return Y
