"""Seeded synthetic inputs for the InfiniGen rehearsal path.

This module only draws random tensors with the shapes and distributions of the
paper's OPT / Llama-2 decode workloads (Section 5.1: models, FP16 KV cache,
partial weight ratio 0.3, alpha 4 / 5).  It holds none of the method's
arithmetic: no skewing, no index generation, no scoring, no attention.  Both
the CPU oracle and the HIP path consume the arrays it returns.

Every tensor of workload ``c`` is drawn from ``numpy.random.default_rng(1000*c + k)``
where ``k`` is the tensor's slot in ``_SLOT``; a per-layer offset keeps distinct
layers distinct.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

_SLOT = {"Wq": 0, "Wk": 1, "Xcal": 2, "x": 3, "x_noise": 4, "K": 5, "V": 6,
         "heavy": 7, "bq": 8, "k_new": 9, "v_new": 10}


@dataclass(frozen=True)
class Workload:
    """Shape and distribution parameters of one synthetic decode layer."""
    cfg: int                 # seed family (1..5 are the documented workloads)
    name: str
    B: int                   # sequences in the batch
    H: int                   # attention heads
    d: int                   # head dimension
    N: int                   # cached tokens per sequence
    dtype: str               # "f32" or "f16": storage type of x, weights, K, V
    ratio: float             # partial weight ratio (Section 5.1: 0.3)
    alpha: float             # threshold slack (Section 5.1: 4 for OPT, 5 for Llama-2)
    decay: float             # singular-value decay of the synthetic Wq / Wk
    heavy_count: int         # heavy-hitter tokens per sequence
    heavy_scale: float       # factor applied to their key rows
    recent_window: int = 0   # last tokens whose keys get recent_scale
    recent_scale: float = 1.0
    rope: bool = False       # rotary embedding between projection and skewing
    pool: str = "hbm"        # "hbm" or "host": where the full K/V pool lives
    n_cal: int = 512         # rows of the calibration input
    gain: float = 1.0        # logit gain of the calibrated variant (scale = gain / sqrt(d)); 1 = literal
    layers: int = 32         # decoder layers of the model the shape is taken from

    @property
    def D(self) -> int:
        return self.H * self.d

    @property
    def np_dtype(self):
        return np.float32 if self.dtype == "f32" else np.float16


WORKLOADS = {
    1: Workload(1, "cfg1 single layer, CPU-checkable", B=1, H=4, d=64, N=512, dtype="f32",
                ratio=0.3, alpha=4.0, decay=0.9, heavy_count=8, heavy_scale=4.0),
    2: Workload(2, "cfg2 OPT-6.7B-shaped decode layer", B=8, H=32, d=128, N=2048, dtype="f16",
                ratio=0.3, alpha=4.0, decay=0.95, heavy_count=20, heavy_scale=3.0, gain=32.0,
                layers=32),
    3: Workload(3, "cfg3 Llama-2-7B-shaped decode layer", B=16, H=32, d=128, N=4096, dtype="f16",
                ratio=0.3, alpha=5.0, decay=0.95, heavy_count=40, heavy_scale=3.0, rope=True,
                gain=54.0, layers=32),
    4: Workload(4, "cfg4 OPT-30B-shaped decode layer, host KV pool", B=20, H=56, d=128, N=2048,
                dtype="f16", ratio=0.3, alpha=4.0, decay=0.95, heavy_count=20, heavy_scale=3.0,
                pool="host", gain=40.0, layers=48),
    5: Workload(5, "cfg5 Llama-2-13B-shaped long context, host KV pool", B=4, H=40, d=128,
                N=32768, dtype="f16", ratio=0.2, alpha=5.0, decay=0.95, heavy_count=163,
                heavy_scale=4.0, recent_window=256, recent_scale=2.0, rope=True, pool="host",
                gain=40.0, layers=40),
}


def shrink(w: Workload, **kw) -> Workload:
    """Same recipe at a smaller (or otherwise altered) shape; used by parity tests."""
    return replace(w, **kw)


def _rng(w: Workload, slot: str, layer: int = 0) -> np.random.Generator:
    return np.random.default_rng(1000 * w.cfg + _SLOT[slot] + 100003 * layer)


def _orthogonal(rng: np.random.Generator, n: int) -> np.ndarray:
    """Random orthogonal matrix: Q factor of a Gaussian matrix, signs fixed by R's diagonal."""
    g = rng.standard_normal((n, n))
    q, r = np.linalg.qr(g)
    return q * np.sign(np.diag(r))[None, :]


def projection_weight(w: Workload, which: str) -> np.ndarray:
    """W = U diag(decay^i) V^T, float32 [D, D] (y = x @ W)."""
    rng = _rng(w, which)
    D = w.D
    U = _orthogonal(rng, D)
    V = _orthogonal(rng, D)
    s = w.decay ** np.arange(D, dtype=np.float64)
    return ((U * s[None, :]) @ V.T).astype(np.float32)


def calibration_input(w: Workload) -> np.ndarray:
    """Sample input rows for the offline pass, float32 [n_cal, D] ~ N(0,1)."""
    return _rng(w, "Xcal").standard_normal((w.n_cal, w.D), dtype=np.float32)


def attention_input(w: Workload, layer: int = 0) -> np.ndarray:
    """Layer-normalised attention input of the previous layer, [B, D] ~ N(0,1)."""
    return _rng(w, "x", layer).standard_normal((w.B, w.D), dtype=np.float32)


def next_layer_input(w: Workload, x: np.ndarray, layer: int = 0, noise: float = 0.3) -> np.ndarray:
    """The next layer's own input: x plus seeded noise (Table 1: consecutive inputs are similar)."""
    e = _rng(w, "x_noise", layer).standard_normal(x.shape, dtype=np.float32)
    return (x + noise * e).astype(np.float32)


def heavy_positions(w: Workload, layer: int = 0) -> np.ndarray:
    """Heavy-hitter token positions, int64 [B, heavy_count], shared by all heads of a sequence."""
    rng = _rng(w, "heavy", layer)
    return np.stack([np.sort(rng.choice(w.N, size=min(w.heavy_count, w.N), replace=False))
                     for _ in range(w.B)])


def key_row_gain(w: Workload, layer: int = 0) -> np.ndarray:
    """Per-token factor on key rows, float32 [B, N]: heavy hitters and the recent window."""
    g = np.ones((w.B, w.N), dtype=np.float32)
    hp = heavy_positions(w, layer)
    for b in range(w.B):
        g[b, hp[b]] *= w.heavy_scale
    if w.recent_window > 0:
        g[:, max(0, w.N - w.recent_window):] *= w.recent_scale
    return g


def kv_cache(w: Workload, layer: int = 0):
    """Keys and values of the cached tokens, float32 [B, H, N, d] each.

    K ~ N(0,1) with heavy-hitter / recent rows scaled by key_row_gain; V ~ N(0,1).
    """
    K = _rng(w, "K", layer).standard_normal((w.B, w.H, w.N, w.d), dtype=np.float32)
    V = _rng(w, "V", layer).standard_normal((w.B, w.H, w.N, w.d), dtype=np.float32)
    K *= key_row_gain(w, layer)[:, None, :, None]
    return K, V


def new_token_kv(w: Workload, layer: int = 0):
    """Key and value of the token being decoded, float32 [B, H, d] each."""
    k = _rng(w, "k_new", layer).standard_normal((w.B, w.H, w.d), dtype=np.float32)
    v = _rng(w, "v_new", layer).standard_normal((w.B, w.H, w.d), dtype=np.float32)
    return k, v


def query_bias(w: Workload) -> np.ndarray:
    """Optional projection bias, float32 [D] ~ 0.1 N(0,1)."""
    return (0.1 * _rng(w, "bq").standard_normal(w.D)).astype(np.float32)


def quantise(a: np.ndarray, w: Workload) -> np.ndarray:
    """Round to the workload's storage dtype (the bits both sides read)."""
    return np.ascontiguousarray(a.astype(w.np_dtype))
