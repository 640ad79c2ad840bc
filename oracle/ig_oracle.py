"""ctypes front end of the CPU oracle (oracle/ig_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
CPU-baseline leg, never by the product package.  All arrays are float32 / int32 numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ig_oracle.c")
_LIB = os.path.join(_HERE, "libig_oracle.so")
_lib = None

OK, EINVAL, ENOCONV, ENOMEM = 0, 1, 2, 3


def build_sanitized(out_dir: str, cc: str) -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer, built with `cc` (the
    clang that builds the library under test, so that one sanitizer runtime serves both)."""
    os.makedirs(out_dir, exist_ok=True)
    lib = os.path.join(out_dir, "libig_oracle.so")
    subprocess.check_call([cc, "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-Wall", "-fsanitize=address",
                           "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-shared-libsan",
                           "-o", lib, _SRC, "-lm"])
    return lib


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (single-threaded, no fast-math).  IG_ORACLE_LIBRARY names an
    already built copy to load instead (the sanitized one)."""
    if os.environ.get("IG_ORACLE_LIBRARY"):
        return os.environ["IG_ORACLE_LIBRARY"]
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-o", _LIB,
                               _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _f(a):
    if a is None:
        return None
    assert a.dtype == np.float32 and a.flags.c_contiguous, (a.dtype, a.flags.c_contiguous)
    return a.ctypes.data_as(ctypes.c_void_p)


def _i(a):
    if a is None:
        return None
    assert a.dtype == np.int32 and a.flags.c_contiguous
    return a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _check(rc, what, allow=()):
    if rc != OK and rc not in allow:
        raise RuntimeError(f"oracle {what} failed with code {rc}")
    return rc


def skew(Wq, Wk, Qcal, H, bq=None, bk=None):
    """Offline skewing. Returns dict(A [H,d,d], sigma [H,d], Wq_s, Wk_s, bq_s, bk_s, rc)."""
    Qcal = _f32(Qcal)
    n_cal, D = Qcal.shape
    d = D // H
    Wq, Wk, bq, bk = _f32(Wq), _f32(Wk), _f32(bq), _f32(bk)
    A = np.zeros((H, d, d), np.float32)
    sigma = np.zeros((H, d), np.float32)
    Wq_s = np.zeros((D, D), np.float32) if Wq is not None else None
    Wk_s = np.zeros((D, D), np.float32) if Wk is not None else None
    bq_s = np.zeros(D, np.float32) if bq is not None else None
    bk_s = np.zeros(D, np.float32) if bk is not None else None
    rc = _load().igo_skew(D, H, n_cal, _f(Wq), _f(Wk), _f(bq), _f(bk), _f(Qcal), _f(A), _f(sigma),
                          _f(Wq_s), _f(Wk_s), _f(bq_s), _f(bk_s))
    _check(rc, "skew", allow=(ENOCONV,))
    return dict(A=A, sigma=sigma, Wq_s=Wq_s, Wk_s=Wk_s, bq_s=bq_s, bk_s=bk_s, rc=rc)


def apply_skew(X, A):
    """Y[..., head h] = X[..., head h] @ A_h for X [..., H*d] (or [..., H, d])."""
    H, d, _ = A.shape
    X = _f32(X)
    shp = X.shape
    X2 = X.reshape(-1, H * d)
    Y = np.zeros_like(X2)
    _check(_load().igo_apply_skew(X2.shape[0], H, d, _f(X2), _f(_f32(A)), _f(Y)), "apply_skew")
    return Y.reshape(shp)


def rope(X, pos, theta=10000.0):
    """Rotate X [rows, H, d] at integer positions pos [rows]."""
    X = _f32(X)
    rows, H, d = X.shape
    pos = _i32(pos)
    assert pos.shape == (rows,)
    Y = np.zeros_like(X)
    _check(_load().igo_rope(rows, H, d, _i(pos), ctypes.c_double(theta), _f(X), _f(Y)), "rope")
    return Y


def partial_index(Qs, Ks, H, ratio):
    """Top floor(ratio*d) columns per head by summed |Q~| (+ |K~|). Returns idx [H,r] ascending."""
    Qs, Ks = _f32(Qs), _f32(Ks)
    n, D = Qs.shape
    d = D // H
    r = ctypes.c_int32(0)
    _check(_load().igo_partial_index(H, d, n, _f(Qs), _f(Ks), ctypes.c_double(ratio), None,
                                     ctypes.byref(r)), "partial_index(r)")
    idx = np.zeros((H, r.value), np.int32)
    _check(_load().igo_partial_index(H, d, n, _f(Qs), _f(Ks), ctypes.c_double(ratio), _i(idx),
                                     ctypes.byref(r)), "partial_index")
    return idx


def project(x, Wq_s, idx, bq_s=None):
    """q_p [B,H,r] = x @ Wq_s[:, kept columns] (+ bias)."""
    x, Wq_s, idx, bq_s = _f32(x), _f32(Wq_s), _i32(idx), _f32(bq_s)
    B, D = x.shape
    H, r = idx.shape
    q_p = np.zeros((B, H, r), np.float32)
    _check(_load().igo_project(B, H, D // H, r, _f(x), _f(Wq_s), _f(bq_s), _i(idx), _f(q_p)),
           "project")
    return q_p


def project_rope(x, Wq, pos, A, idx, bq=None, theta=10000.0):
    x, Wq, A, idx, bq, pos = _f32(x), _f32(Wq), _f32(A), _i32(idx), _f32(bq), _i32(pos)
    B, D = x.shape
    H, r = idx.shape
    q_p = np.zeros((B, H, r), np.float32)
    _check(_load().igo_project_rope(B, H, D // H, r, _f(x), _f(Wq), _f(bq), _i(pos),
                                    ctypes.c_double(theta), _f(A), _i(idx), _f(q_p)),
           "project_rope")
    return q_p


def scan(q_p, Kt, idx, scale, N=None):
    """s [B,H,N] = scale * q_p . Kt[..., kept columns]; Kt [B,H,N_cap,d]."""
    q_p, Kt, idx = _f32(q_p), _f32(Kt), _i32(idx)
    B, H, N_cap, d = Kt.shape
    N = N_cap if N is None else N
    r = idx.shape[1]
    s = np.zeros((B, H, N), np.float32)
    _check(_load().igo_scan(B, H, N, N_cap, d, r, ctypes.c_float(scale), _f(q_p), _f(Kt), _i(idx),
                            _f(s)), "scan")
    return s


def select(s, alpha, stride=None):
    """Per-head threshold selection. Returns (sel_idx [B*H, stride] int32, sel_cnt [B*H])."""
    s = _f32(s)
    B, H, N = s.shape
    stride = N if stride is None else stride
    sel_idx = np.full((B * H, stride), -1, np.int32)
    sel_cnt = np.zeros(B * H, np.int32)
    _check(_load().igo_select(B, H, N, _f(s), ctypes.c_float(alpha), _i(sel_idx), stride,
                              _i(sel_cnt)), "select")
    return sel_idx, sel_cnt


def select_equalized(s, alpha, max_frac=0.2, stride=None):
    """Head-equalised selection: every head of a sequence keeps the same number of tokens.

    Returns (sel_idx [B*H, stride] int32 ascending, sel_cnt [B*H], n_eq [B])."""
    s = _f32(s)
    B, H, N = s.shape
    stride = N if stride is None else stride
    sel_idx = np.full((B * H, stride), -1, np.int32)
    sel_cnt = np.zeros(B * H, np.int32)
    n_eq = np.zeros(B, np.int32)
    _check(_load().igo_select_equalized(B, H, N, _f(s), ctypes.c_float(alpha),
                                        ctypes.c_double(max_frac), _i(sel_idx), stride,
                                        _i(sel_cnt), _i(n_eq)), "select_equalized")
    return sel_idx, sel_cnt, n_eq


def pool_touch(counters, sel_idx, sel_cnt, N, counter_max=255):
    """Counter policy: +1 for every prefetched slot (saturating), halve a pool whose counter saturates.
    counters int32 [B*H, N_cap], updated in place."""
    assert counters.dtype == np.int32 and counters.flags.c_contiguous
    sel_idx, sel_cnt = _i32(sel_idx), _i32(sel_cnt)
    BH, N_cap = counters.shape
    _check(_load().igo_pool_touch(BH, N, N_cap, _i(sel_idx), sel_idx.shape[1], _i(sel_cnt),
                                  _i(counters), counter_max), "pool_touch")
    return counters


def pool_victim(counters, N):
    """Slot with the smallest count among the first N of every pool (ties: the lowest slot)."""
    counters = _i32(counters)
    BH, N_cap = counters.shape
    victim = np.zeros(BH, np.int32)
    _check(_load().igo_pool_victim(BH, N, N_cap, _i(counters), _i(victim)), "pool_victim")
    return victim


def pool_touch_lru(stamps, sel_idx, sel_cnt, N, now):
    """LRU comparison policy: every prefetched slot's last-use stamp becomes `now`.
    stamps int32 [B*H, N_cap], updated in place."""
    assert stamps.dtype == np.int32 and stamps.flags.c_contiguous
    sel_idx, sel_cnt = _i32(sel_idx), _i32(sel_cnt)
    BH, N_cap = stamps.shape
    _check(_load().igo_pool_touch_lru(BH, N, N_cap, _i(sel_idx), sel_idx.shape[1], _i(sel_cnt),
                                      _i(stamps), int(now)), "pool_touch_lru")
    return stamps


def pool_victim_oldest(stamps, N):
    """Slot with the oldest stamp among the first N of every pool (ties: the lowest slot): the FIFO
    victim for insertion stamps, the LRU victim for last-use stamps."""
    stamps = _i32(stamps)
    BH, N_cap = stamps.shape
    victim = np.zeros(BH, np.int32)
    _check(_load().igo_pool_victim_oldest(BH, N, N_cap, _i(stamps), _i(victim)), "pool_victim_oldest")
    return victim


def gather(pool, sel_idx, sel_cnt):
    """Rows pool[bh, sel_idx[bh, j]] -> out [B*H, stride, d] (zeros beyond the count)."""
    pool, sel_idx, sel_cnt = _f32(pool), _i32(sel_idx), _i32(sel_cnt)
    d = pool.shape[-1]
    N_cap = pool.shape[-2]
    BH, stride = sel_idx.shape
    pool2 = pool.reshape(BH, N_cap, d)
    out = np.zeros((BH, stride, d), np.float32)
    _check(_load().igo_gather(BH, N_cap, d, _f(pool2), _i(sel_idx), stride, _i(sel_cnt), _f(out)),
           "gather")
    return out


def attend(q, K_sel, V_sel, sel_cnt, scale, k_new=None, v_new=None):
    """Decode attention over the gathered rows. q [B*H, d] (or [B,H,d]); returns [B*H, d]."""
    K_sel, V_sel, sel_cnt = _f32(K_sel), _f32(V_sel), _i32(sel_cnt)
    BH, stride, d = K_sel.shape
    q = _f32(q).reshape(BH, d)
    k_new = None if k_new is None else _f32(k_new).reshape(BH, d)
    v_new = None if v_new is None else _f32(v_new).reshape(BH, d)
    out = np.zeros((BH, d), np.float32)
    _check(_load().igo_attend(BH, d, stride, ctypes.c_float(scale), _f(q), _f(K_sel), _f(V_sel),
                              _i(sel_cnt), _f(k_new), _f(v_new), _f(out)), "attend")
    return out
