"""Shared test plumbing: builds one layer's inputs from a workload and runs the oracle on them.

Inputs that both sides read are rounded to the workload's storage dtype first; the oracle gets
their exact float32 upcasts.  The setup steps (skew, index generation, skewed keys) are done with
the oracle, so the HIP path is fed oracle-side inputs only.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

import ig_workloads as wl
from oracle import ig_oracle as o


@dataclass
class Case:
    w: wl.Workload
    scale: float
    r: int
    idx: np.ndarray          # [H, r] int32
    A: np.ndarray            # [H, d, d] float32
    A_p: np.ndarray          # [H, d, r] float32
    W_in: np.ndarray         # storage dtype [D, D]: skewed W~q (folded) or original Wq (rope)
    bias_full: np.ndarray    # float32 [D] or None (skewed bias in folded mode)
    bias_in: np.ndarray      # float32 [H*r] (folded) / [D] (rope) or None
    x: np.ndarray            # storage dtype [B, D]
    pos: np.ndarray          # int32 [B]
    Kt: np.ndarray           # storage dtype [B, H, N_cap, d] skewed keys
    V: np.ndarray            # storage dtype [B, H, N_cap, d]
    q: np.ndarray            # storage dtype [B, H, d] real skewed query of the layer
    k_new: np.ndarray
    v_new: np.ndarray
    N: int
    N_cap: int

    def f32(self, name):
        return np.ascontiguousarray(getattr(self, name), dtype=np.float32)


def _skew_keys(K: np.ndarray, A: np.ndarray) -> np.ndarray:
    """K~ = K A_h with the oracle, one sequence per thread for large caches (sequences are
    independent; the C routine itself is single-threaded and untouched)."""
    B = K.shape[0]
    if K.size < (1 << 24) or B == 1:
        return o.apply_skew(K.transpose(0, 2, 1, 3), A).transpose(0, 2, 1, 3)
    from concurrent.futures import ThreadPoolExecutor
    import os
    one = lambda b: o.apply_skew(np.ascontiguousarray(K[b:b + 1].transpose(0, 2, 1, 3)), A)   # noqa: E731
    with ThreadPoolExecutor(min(B, os.cpu_count() or 1, 16)) as ex:
        parts = list(ex.map(one, range(B)))
    return np.concatenate(parts, axis=0).transpose(0, 2, 1, 3)


def make_case(w: wl.Workload, gain: float = 1.0, layer: int = 0, bias: bool = False,
              N_cap: int | None = None, all_columns: bool = False, use_keys_for_index: bool = False) -> Case:
    N_cap = w.N if N_cap is None else N_cap
    Wq = wl.projection_weight(w, "Wq")
    Xcal = wl.calibration_input(w)
    bq = wl.query_bias(w) if bias else None
    Qcal = Xcal @ Wq + (bq if bias else 0.0)
    if w.rope:
        Qcal = o.rope(Qcal.reshape(w.n_cal, w.H, w.d), np.arange(w.n_cal, dtype=np.int32)).reshape(w.n_cal, w.D)
    sk = o.skew(Wq, None, Qcal, w.H, bq=bq)
    A = sk["A"]
    K, V = wl.kv_cache(w, layer)                                  # K: (rotated) keys before skewing
    Kt = _skew_keys(K, A)
    Qs_cal = o.apply_skew(Qcal, A)
    if all_columns:
        idx = np.tile(np.arange(w.d, dtype=np.int32), (w.H, 1))
    else:
        Ks_cal = None
        if use_keys_for_index:
            Ks_cal = Kt[0].transpose(1, 0, 2).reshape(w.N, w.D)[: w.n_cal]
            Qs_cal = Qs_cal[: Ks_cal.shape[0]]
        idx = o.partial_index(Qs_cal, Ks_cal, w.H, w.ratio)
    r = idx.shape[1]
    A_p = np.ascontiguousarray(np.stack([A[h][:, idx[h]] for h in range(w.H)]), dtype=np.float32)
    x = wl.quantise(wl.attention_input(w, layer), w)
    x_next = wl.next_layer_input(w, x.astype(np.float32), layer)
    pos = np.full(w.B, w.N, np.int32)
    if w.rope:
        W_in = wl.quantise(Wq, w)
        bias_full = bq
        bias_in = bq
        qfull = (x_next @ W_in.astype(np.float32) + (bq if bias else 0.0)).reshape(w.B, w.H, w.d)
        q = o.apply_skew(o.rope(qfull, pos), A)
    else:
        W_in = wl.quantise(sk["Wq_s"], w)
        bias_full = sk["bq_s"]
        cols = (np.arange(w.H)[:, None] * w.d + idx).reshape(-1)
        bias_in = np.ascontiguousarray(bias_full[cols]) if bias else None
        q = (x_next @ W_in.astype(np.float32) + (bias_full if bias else 0.0)).reshape(w.B, w.H, w.d)
    Kt_q = np.zeros((w.B, w.H, N_cap, w.d), w.np_dtype)
    V_q = np.zeros((w.B, w.H, N_cap, w.d), w.np_dtype)
    Kt_q[:, :, : w.N] = wl.quantise(Kt, w)
    V_q[:, :, : w.N] = wl.quantise(V, w)
    if N_cap > w.N:       # rows beyond N hold junk that must never be read into a result
        Kt_q[:, :, w.N:] = 7.0
        V_q[:, :, w.N:] = -3.0
    kn, vn = wl.new_token_kv(w, layer)
    return Case(w=w, scale=gain / np.sqrt(w.d), r=r, idx=idx, A=A, A_p=A_p, W_in=W_in,
                bias_full=bias_full if bias else None, bias_in=bias_in if bias else None, x=x,
                pos=pos, Kt=Kt_q, V=V_q, q=wl.quantise(q, w), k_new=wl.quantise(kn, w),
                v_new=wl.quantise(vn, w), N=w.N, N_cap=N_cap)


@dataclass
class OracleResult:
    q_p: np.ndarray       # [B,H,r]
    s: np.ndarray         # [B,H,N]
    sel_idx: np.ndarray   # [B*H, N]
    sel_cnt: np.ndarray
    K_sel: np.ndarray
    V_sel: np.ndarray
    out: np.ndarray       # [B*H, d]
    out_new: np.ndarray   # with the new-token row


def _run_oracle_rows(c: Case, alpha: float, attend: bool, b0: int, b1: int) -> OracleResult:
    """The oracle on sequences b0 .. b1-1 of the case."""
    w = c.w
    x, pos = c.f32("x")[b0:b1], c.pos[b0:b1]
    if w.rope:
        q_p = o.project_rope(x, c.f32("W_in"), pos, c.A, c.idx, bq=c.bias_full)
    else:
        q_p = o.project(x, c.f32("W_in"), c.idx, bq_s=c.bias_full)
    Kt = np.ascontiguousarray(c.Kt[b0:b1], dtype=np.float32)
    s = o.scan(q_p, Kt, c.idx, c.scale, N=c.N)
    sel_idx, sel_cnt = o.select(s, alpha)
    if not attend:
        return OracleResult(q_p, s, sel_idx, sel_cnt, None, None, None, None)
    V = np.ascontiguousarray(c.V[b0:b1], dtype=np.float32)
    q = np.ascontiguousarray(c.q[b0:b1], dtype=np.float32)
    K_sel = o.gather(Kt, sel_idx, sel_cnt)
    V_sel = o.gather(V, sel_idx, sel_cnt)
    out = o.attend(q, K_sel, V_sel, sel_cnt, c.scale)
    kn = np.ascontiguousarray(c.k_new[b0:b1], dtype=np.float32)
    vn = np.ascontiguousarray(c.v_new[b0:b1], dtype=np.float32)
    out_new = o.attend(q, K_sel, V_sel, sel_cnt, c.scale, kn, vn)
    return OracleResult(q_p, s, sel_idx, sel_cnt, K_sel, V_sel, out, out_new)


def run_oracle(c: Case, alpha: float | None = None, attend: bool = True) -> OracleResult:
    """The oracle on the whole case.  Sequences are independent, so large cases run one sequence per
    thread (the C oracle itself stays single-threaded and untouched; ctypes releases the GIL)."""
    w = c.w
    alpha = w.alpha if alpha is None else alpha
    if w.B * w.H * c.N < (1 << 22) or w.B == 1:
        return _run_oracle_rows(c, alpha, attend, 0, w.B)
    from concurrent.futures import ThreadPoolExecutor
    import os
    with ThreadPoolExecutor(min(w.B, os.cpu_count() or 1, 16)) as ex:
        parts = list(ex.map(lambda b: _run_oracle_rows(c, alpha, attend, b, b + 1), range(w.B)))
    cat = lambda name: (None if getattr(parts[0], name) is None   # noqa: E731
                        else np.concatenate([getattr(p, name) for p in parts], axis=0))
    return OracleResult(*[cat(n) for n in ("q_p", "s", "sel_idx", "sel_cnt", "K_sel", "V_sel", "out", "out_new")])


def selected_fraction(res: OracleResult, N: int) -> float:
    return float(res.sel_cnt.mean()) / N


def compare_selection(gpu_idx, gpu_cnt, res: OracleResult, alpha: float, band: float = 1e-3):
    """Index sets must be identical except for tokens whose oracle score lies within `band` of the
    oracle threshold.  Returns the number of in-band disagreements; raises on any other."""
    BH, N = res.s.reshape(-1, res.s.shape[-1]).shape
    s = res.s.reshape(BH, N)
    slack = 0
    for i in range(BH):
        g = gpu_idx[i, : gpu_cnt[i]]
        assert np.all(np.diff(g) > 0), f"list {i} is not strictly ascending"
        assert g.size == 0 or (g[0] >= 0 and g[-1] < N)
        ref = res.sel_idx[i, : res.sel_cnt[i]]
        diff = np.setxor1d(g, ref)
        if diff.size:
            thr = np.float32(s[i].max()) - np.float32(alpha)
            bad = diff[np.abs(s[i, diff] - thr) > band]
            assert bad.size == 0, (f"list {i}: tokens {bad[:8]} differ outside the band "
                                   f"(scores {s[i, bad[:8]]}, threshold {thr})")
            slack += diff.size
    return slack
