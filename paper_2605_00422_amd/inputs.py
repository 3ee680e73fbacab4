"""Seeded synthetic inputs shaped like the paper's layers.

This module only draws random tensors and rounds them to their storage grids; it holds none
of the method's arithmetic, so both the CPU oracle's callers and the HIP path's callers can
use it.  The recipe stands in for the LLaMA / Qwen3 linear layers the paper quantizes
(paper Sec. 4, Table 1), whose weights are not available here:

  X      i.i.d. Student-t (df = 3) fp32, a few "outlier" channels (columns) scaled up for
         every token (heavy tails and outlier channels: paper Sec. 1, Fig. 2(a)), then
         rounded to bf16 when the layer takes bf16 activations;
  R1,R2  Q factor of the QR decomposition of a seeded Gaussian matrix (fp64), sign-fixed,
         stored fp32 (the paper's factors are orthogonal, Sec. 3.1);
  W_rot  N(0, 0.02^2) fp32: the weight already in rotated, PSP-corrected coordinates;
  U, V   N(0, 0.01^2) rounded to fp16: the PSP factors (Sec. 3.2: M = A B; V = A, U = B^T).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass(frozen=True)
class LayerConfig:
    name: str
    M: int
    K: int
    n1: int
    n2: int
    N: int
    r: int
    x_dtype: str = "bf16"          # "f32" or "bf16"
    outlier_channels: int = 0      # number of scaled columns
    outlier_scale: float = 1.0
    seed: int = 0


# Kronecker pairs (n1, n2) of the block widths used below, as the paper's Algorithm 1 gives them
# (App. A.1): written out, so that this module holds none of the method's steps.  The tests hold
# them against both the oracle's and the library's implementation of the algorithm.
KRON_PAIRS = {4096: (64, 64), 8192: (128, 64), 11008: (128, 86), 28672: (224, 128)}


def _pct(K: int, frac: float) -> int:
    return int(round(frac * K))


# The five workload families.  Factor pairs for 0-3 are read literally from the task's
# configuration list (n1 x n2); family 4 uses the near-square pair.
CONFIGS: dict[str, LayerConfig] = {
    "cfg0_tiny": LayerConfig("cfg0_tiny", 16, 512, 16, 32, 512, 8, "f32", 4, 20.0),
    "cfg1_decode7b": LayerConfig("cfg1_decode7b", 1, 4096, 64, 64, 11008, 32, "bf16", 4, 20.0),
    "cfg2_qwen32b_up_m16": LayerConfig("cfg2_qwen32b_up_m16", 16, 5120, 64, 80, 25600, 64, "bf16",
                                       _pct(5120, 0.01), 50.0),
    "cfg3_qwen32b_down_m2048": LayerConfig("cfg3_qwen32b_down_m2048", 2048, 25600, 160, 160, 5120, 64,
                                           "bf16", _pct(25600, 0.01), 50.0),
}


def block70b_configs(M: int) -> list[LayerConfig]:
    """70B-shaped decoder block: hidden 8192, intermediate 28672, GQA kv width 1024."""
    h, inter, kv = 8192, 28672, 1024
    out = []
    for nm, K, N in (("q", h, h), ("k", h, kv), ("v", h, kv), ("o", h, h),
                     ("gate", h, inter), ("up", h, inter), ("down", inter, h)):
        n1, n2 = KRON_PAIRS[K]
        out.append(LayerConfig(f"cfg4_70b_{nm}_m{M}", M, K, n1, n2, N, 64, "bf16",
                               _pct(K, 0.01), 50.0))
    return out


def block7b_configs(M: int) -> list[LayerConfig]:
    """7B-shaped decoder block (the model of cfg1, whose layer is this block's gate/up projection):
    hidden 4096, intermediate 11008; Kronecker pairs by Algorithm 1 (11008 = 128 x 86).
    "qkv" and "gateup" are the projections that read the same activations packed as one layer
    (rows stacked, one rotation pair, the ranks of the parts added up): one rotation and one GEMM
    launch serve all of them."""
    h, inter = 4096, 11008
    out = []
    for nm, K, N, r in (("q", h, h, 32), ("gate", h, inter, 32), ("down", inter, h, 32),
                        ("qkv", h, 3 * h, 96), ("gateup", h, 2 * inter, 64)):
        n1, n2 = KRON_PAIRS[K]
        out.append(LayerConfig(f"cfg1_7b_{nm}_m{M}", M, K, n1, n2, N, r, "bf16", _pct(K, 0.01), 50.0))
    return out


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) & np.uint32(0xFFFF0000)).view(np.float32)


def random_orthogonal(rng: np.random.Generator, n: int) -> np.ndarray:
    g = rng.standard_normal((n, n))
    q, rr = np.linalg.qr(g)
    q = q * np.sign(np.diag(rr))[None, :]
    return q.astype(np.float32)


@dataclass
class LayerData:
    cfg: LayerConfig
    X: np.ndarray          # (M,K) fp32, on the bf16 grid when cfg.x_dtype == "bf16"
    R1: np.ndarray         # (n1,n1) fp32
    R2: np.ndarray         # (n2,n2) fp32
    W: np.ndarray          # (N,K) fp32
    U: np.ndarray          # (K,r) fp32 on the fp16 grid
    V: np.ndarray          # (N,r) fp32 on the fp16 grid
    outlier_idx: np.ndarray = field(default_factory=lambda: np.zeros(0, dtype=np.int64))


def make_activations(cfg: LayerConfig, rng: np.random.Generator, M: int | None = None):
    M = cfg.M if M is None else M
    X = rng.standard_t(3.0, size=(M, cfg.K)).astype(np.float32)
    idx = np.zeros(0, dtype=np.int64)
    if cfg.outlier_channels > 0:
        idx = np.sort(rng.choice(cfg.K, size=cfg.outlier_channels, replace=False))
        X[:, idx] *= np.float32(cfg.outlier_scale)
    if cfg.x_dtype == "bf16":
        X = round_to_bf16(X)
    return X, idx


def make_layer(cfg: LayerConfig, with_activations: bool = True) -> LayerData:
    """Draw order (one generator, fixed): R1, R2, W, U, V, then X."""
    rng = np.random.default_rng(cfg.seed)
    R1 = random_orthogonal(rng, cfg.n1)
    R2 = random_orthogonal(rng, cfg.n2)
    W = (rng.standard_normal((cfg.N, cfg.K), dtype=np.float32) * np.float32(0.02))
    U = (rng.standard_normal((cfg.K, cfg.r)) * 0.01).astype(np.float16).astype(np.float32)
    V = (rng.standard_normal((cfg.N, cfg.r)) * 0.01).astype(np.float16).astype(np.float32)
    if with_activations:
        X, idx = make_activations(cfg, rng)
    else:
        X, idx = np.zeros((0, cfg.K), dtype=np.float32), np.zeros(0, dtype=np.int64)
    return LayerData(cfg, X, R1, R2, W, U, V, idx)


def shifted_weights(d: LayerData) -> np.ndarray:
    """The layer's weights with a seeded offset per output channel (N(0, 0.01^2), half a standard
    deviation of the weights): input of the binarization with the row shift, which a zero-mean
    Gaussian matrix would not exercise.  A generator of its own, so that the draws of make_layer
    stay as they are."""
    rng = np.random.default_rng(1000 + d.cfg.seed)
    return (d.W + rng.normal(0.0, 0.01, size=(d.cfg.N, 1))).astype(np.float32)
