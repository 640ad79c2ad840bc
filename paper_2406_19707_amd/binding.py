"""Python binding of libinfinigen_hip.so: argument marshalling only.

Every function has the name and argument order of its C entry point in include/infinigen.h.
Tensor arguments are torch tensors (device memory / pinned host memory) or numpy arrays (host
arguments of the offline calls); what crosses the boundary is their address.  There is no fallback:
if the shared library is missing the import of any entry point raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

__all__ = [
    "IG_OK", "IG_EINVAL", "IG_ESHAPE", "IG_EDTYPE", "IG_ECAPACITY", "IG_EHIP", "IG_ENOCONV",
    "IG_ENOMEM", "IG_F32", "IG_F16", "IG_MEM_DEVICE", "IG_MEM_HOST_PINNED", "IG_POLICY_COUNTER", "IG_POLICY_FIFO", "IG_POLICY_LRU", "IG_K_PROJECT",
    "IG_K_FINALIZE", "IG_K_SCAN", "IG_K_SELECT", "IG_K_GATHER", "IG_K_ATTENTION", "IG_K_BUILD",
    "IG_K_COPY", "IG_K_READ", "IG_K_LAYER", "IgDesc", "IgLayerIO", "IgBufferSet", "IgError", "Context", "lib", "lib_path", "ig_skew_offline",
    "ig_partial_index", "ig_apply_skew", "ig_rope_rows", "ig_speculate_host", "ig_wq_bytes", "ig_slab_bytes", "EXPORTS",
]

IG_OK, IG_EINVAL, IG_ESHAPE, IG_EDTYPE, IG_ECAPACITY, IG_EHIP, IG_ENOCONV, IG_ENOMEM = range(8)
IG_F32, IG_F16 = 0, 1
IG_MEM_DEVICE, IG_MEM_HOST_PINNED = 0, 1
IG_POLICY_COUNTER, IG_POLICY_FIFO, IG_POLICY_LRU = 0, 1, 2
(IG_K_PROJECT, IG_K_FINALIZE, IG_K_SCAN, IG_K_SELECT, IG_K_GATHER, IG_K_ATTENTION, IG_K_BUILD,
 IG_K_COPY, IG_K_READ, IG_K_LAYER) = range(10)

# every symbol include/infinigen.h declares
EXPORTS = [
    "ig_create", "ig_destroy", "ig_last_error", "ig_reserve", "ig_workspace_bytes", "ig_check_status",
    "ig_skew_offline", "ig_apply_skew", "ig_rope_rows",
    "ig_partial_index", "ig_skew_device", "ig_partial_index_device", "ig_wq_bytes", "ig_wq_build", "ig_slab_bytes",
    "ig_slab_build", "ig_append_token",
    "ig_pool_touch", "ig_pool_victim", "ig_pool_replace", "ig_pool_touch_policy", "ig_pool_replace_policy",
    "ig_speculate", "ig_project", "ig_scan_select", "ig_project_indexed", "ig_speculate_indexed",
    "ig_speculate_host", "ig_speculate_equalized", "ig_equalize_heads", "ig_gather_kv", "ig_sparse_attention", "ig_sparse_attention_static",
    "ig_sparse_attention_indexed", "ig_gather_attention", "ig_layer_step", "ig_decode_step_overlapped", "ig_set_wait_limit", "ig_profile_begin", "ig_profile_end", "ig_profile_read",
    "ig_copy_bytes", "ig_read_bytes",
]


class IgDesc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("d", ctypes.c_int32),
                ("r", ctypes.c_int32), ("N", ctypes.c_int32), ("N_cap", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("scale", ctypes.c_float), ("alpha", ctypes.c_float),
                ("rope", ctypes.c_int32), ("rope_theta", ctypes.c_float)]

    def __init__(self, B, H, d, r, N, N_cap=None, dtype=IG_F16, scale=1.0, alpha=4.0, rope=0,
                 rope_theta=10000.0):
        super().__init__(B, H, d, r, N, N if N_cap is None else N_cap, dtype, scale, alpha, rope,
                         rope_theta)


class IgLayerIO(ctypes.Structure):
    """One layer's tensors for ig_decode_step_overlapped (device / pinned-host addresses)."""
    _fields_ = [(n, ctypes.c_void_p) for n in ("x", "slab", "q", "Kpool", "Vpool", "k_new", "v_new", "out")]


class IgBufferSet(ctypes.Structure):
    """One rotating set of list and row buffers for ig_decode_step_overlapped."""
    _fields_ = [(n, ctypes.c_void_p) for n in ("sel_idx", "sel_cnt", "K_sel", "V_sel")]


class IgError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"infinigen error {code}: {message}")
        self.code = code


def lib_path() -> str:
    """The built library beside this file; IG_LIBRARY names another build of it (the host-sanitized
    one of the CPU test suite)."""
    if os.environ.get("IG_LIBRARY"):
        return os.environ["IG_LIBRARY"]
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libinfinigen_hip.so")


_lib = None
_vp, _i32, _f32, _sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
_dp = ctypes.POINTER(IgDesc)


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise FileNotFoundError(f"{path} is missing: build it with "
                                    "`python paper_2406_19707_amd/build.py` (there is no fallback)")
        L = ctypes.CDLL(path)
        sig = {
            "ig_create": (ctypes.c_int, [ctypes.c_int, ctypes.POINTER(_vp)]),
            "ig_destroy": (ctypes.c_int, [_vp]),
            "ig_last_error": (ctypes.c_char_p, [_vp]),
            "ig_reserve": (ctypes.c_int, [_vp, _dp]),
            "ig_workspace_bytes": (ctypes.c_size_t, [_vp]),
            "ig_check_status": (ctypes.c_int, [_vp]),
            "ig_skew_offline": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.c_int, ctypes.c_int] + [_vp] * 11),
            "ig_apply_skew": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, _vp, _vp, _vp]),
            "ig_rope_rows": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, _vp, ctypes.c_double, _vp]),
            "ig_partial_index": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, _vp, _vp,
                                                ctypes.c_double, _vp, ctypes.POINTER(_i32)]),
            "ig_skew_device": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, _vp, _vp, _vp, _vp]),
            "ig_partial_index_device": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                       ctypes.c_int, _vp, _vp, ctypes.c_double, _vp, _vp]),
            "ig_wq_bytes": (_sz, [_dp]),
            "ig_wq_build": (ctypes.c_int, [_vp, _dp, _vp, _vp, _vp, _vp]),
            "ig_slab_bytes": (_sz, [_dp]),
            "ig_slab_build": (ctypes.c_int, [_vp, _dp, _vp, ctypes.c_int, _vp, _vp, _vp]),
            "ig_append_token": (ctypes.c_int, [_vp, _dp, _vp, _vp, _vp, _vp, _vp, _vp, ctypes.c_int, _vp]),
            "ig_pool_touch": (ctypes.c_int, [_vp, _dp, _vp, _i32, _vp, _vp, _i32, _vp]),
            "ig_pool_victim": (ctypes.c_int, [_vp, _dp, _vp, _vp, _vp]),
            "ig_pool_replace": (ctypes.c_int, [_vp, _dp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, ctypes.c_int, _vp, _vp]),
            "ig_pool_touch_policy": (ctypes.c_int, [_vp, _dp, ctypes.c_int, _vp, _i32, _vp, _vp, _i32, _vp]),
            "ig_pool_replace_policy": (ctypes.c_int, [_vp, _dp, ctypes.c_int, _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                                      ctypes.c_int, _vp, _i32, _vp]),
            "ig_speculate": (ctypes.c_int, [_vp, _dp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp]),
            "ig_project": (ctypes.c_int, [_vp, _dp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
            "ig_scan_select": (ctypes.c_int, [_vp, _dp, _vp, _vp, _vp, _i32, _vp, _vp, _vp]),
            "ig_project_indexed": (ctypes.c_int, [_vp, _dp, _vp, _vp, _vp, _vp, _vp, _vp]),
            "ig_speculate_indexed": (ctypes.c_int, [_vp, _dp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp]),
            "ig_layer_step": (ctypes.c_int, [_vp, _dp] + [_vp] * 13 + [_i32] + [_vp] * 6),
            "ig_speculate_host": (ctypes.c_int, [_vp, _dp, _vp, _vp, _vp, _i32, _vp, _vp, ctypes.c_int]),
            "ig_speculate_equalized": (ctypes.c_int, [_vp, _dp, _vp, _vp, _vp, _vp, _vp, _vp, ctypes.c_double, _vp, _i32,
                                                      _vp, _vp, _vp]),
            "ig_equalize_heads": (ctypes.c_int, [_vp, _dp, _vp, _vp, ctypes.c_double, _vp, _i32, _vp, _vp]),
            "ig_gather_kv": (ctypes.c_int, [_vp, _dp, _vp, _vp, ctypes.c_int, _vp, _i32, _vp, _vp, _vp, _vp]),
            "ig_sparse_attention": (ctypes.c_int, [_vp, _dp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp]),
            "ig_sparse_attention_static": (ctypes.c_int, [_vp, _dp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp]),
            "ig_sparse_attention_indexed": (ctypes.c_int, [_vp, _dp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp]),
            "ig_gather_attention": (ctypes.c_int, [_vp, _dp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
            "ig_decode_step_overlapped": (ctypes.c_int, [_vp, _dp, ctypes.c_int, _vp, _vp, _vp, _vp, _vp, ctypes.c_int,
                                                         ctypes.c_int, _vp, _i32, _vp, _vp]),
            "ig_set_wait_limit": (ctypes.c_int, [_vp, ctypes.c_int64]),
            "ig_profile_begin": (ctypes.c_int, [_vp]),
            "ig_profile_end": (ctypes.c_int, [_vp]),
            "ig_profile_read": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.POINTER(ctypes.c_double),
                                               ctypes.POINTER(_i32)]),
            "ig_copy_bytes": (ctypes.c_int, [_vp, _vp, _vp, _sz, _vp]),
            "ig_read_bytes": (ctypes.c_int, [_vp, _vp, _sz, _vp]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _ptr(t):
    """Address of a torch tensor / numpy array / None / raw int."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        assert t.flags.c_contiguous
        return t.ctypes.data
    assert t.is_contiguous(), "tensors crossing the C ABI must be contiguous"
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _host_f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def ig_wq_bytes(desc: IgDesc) -> int:
    return lib().ig_wq_bytes(ctypes.byref(desc))


def ig_slab_bytes(desc: IgDesc) -> int:
    return lib().ig_slab_bytes(ctypes.byref(desc))


def ig_skew_offline(Wq, Wk, Qcal, H, bq=None, bk=None, ctx=None):
    """Host call. Returns dict(A, sigma, Wq_s, Wk_s, bq_s, bk_s, rc); rc is IG_OK or IG_ENOCONV."""
    Qcal = _host_f32(Qcal)
    n_cal, D = Qcal.shape
    d = D // H
    Wq, Wk, bq, bk = map(_host_f32, (Wq, Wk, bq, bk))
    A = np.zeros((H, d, d), np.float32)
    sigma = np.zeros((H, d), np.float32)
    out = {k: (np.zeros_like(v) if v is not None else None)
           for k, v in (("Wq_s", Wq), ("Wk_s", Wk), ("bq_s", bq), ("bk_s", bk))}
    rc = lib().ig_skew_offline(ctx._h if ctx else None, D, H, n_cal, _ptr(Wq), _ptr(Wk), _ptr(bq),
                               _ptr(bk), _ptr(Qcal), _ptr(A), _ptr(sigma), _ptr(out["Wq_s"]),
                               _ptr(out["Wk_s"]), _ptr(out["bq_s"]), _ptr(out["bk_s"]))
    if rc not in (IG_OK, IG_ENOCONV):
        raise IgError(rc, ctx.last_error() if ctx else "ig_skew_offline")
    return dict(A=A, sigma=sigma, rc=rc, **out)


def ig_apply_skew(X, A, ctx=None):
    """Host call. X [n, H*d], A [H, d, d] -> Y [n, H*d] with every head block multiplied by A_h."""
    X, A = _host_f32(X), _host_f32(A)
    H, d = A.shape[0], A.shape[1]
    n = X.shape[0]
    Y = np.empty_like(X)
    rc = lib().ig_apply_skew(ctx._h if ctx else None, H, d, n, _ptr(X), _ptr(A), _ptr(Y))
    if rc != IG_OK:
        raise IgError(rc, ctx.last_error() if ctx else "ig_apply_skew")
    return Y


def ig_rope_rows(q, pos, theta=10000.0, ctx=None):
    """Host call. q [n, H, d] float32, pos int32 [n] -> rotated copy."""
    q = np.array(q, dtype=np.float32, order="C", copy=True)
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    n, H, d = q.shape
    rc = lib().ig_rope_rows(ctx._h if ctx else None, n, H, d, _ptr(pos), float(theta), _ptr(q))
    if rc != IG_OK:
        raise IgError(rc, ctx.last_error() if ctx else "ig_rope_rows")
    return q


def ig_speculate_host(desc, q_p, slab_host, sel_stride=None, want_scores=False, threads=0, ctx=None):
    """Host call (Section 6.2: speculation on the CPU, partial key cache in host memory).
    q_p: numpy float32 [B,H,r]; slab_host: numpy uint8 / pinned torch tensor holding the slab bytes.
    Returns (sel_idx [B*H, stride] int32, sel_cnt [B*H] int32, scores or None, status)."""
    q_p = _host_f32(q_p)
    BH = desc.B * desc.H
    stride = desc.N if sel_stride is None else sel_stride
    sel_idx = np.full((BH, stride), -1, np.int32)
    sel_cnt = np.zeros(BH, np.int32)
    scores = np.zeros((desc.B, desc.H, desc.N), np.float32) if want_scores else None
    rc = lib().ig_speculate_host(ctx._h if ctx else None, ctypes.byref(desc), _ptr(q_p), _ptr(slab_host),
                                 _ptr(sel_idx), stride, _ptr(sel_cnt), _ptr(scores), threads)
    if rc not in (IG_OK, IG_ECAPACITY):
        raise IgError(rc, ctx.last_error() if ctx else "ig_speculate_host")
    return sel_idx, sel_cnt, scores, rc


def ig_partial_index(Qs, Ks, H, ratio, ctx=None):
    """Host call. Returns idx int32 [H, r]."""
    Qs, Ks = _host_f32(Qs), _host_f32(Ks)
    n, D = Qs.shape
    d = D // H
    r = _i32(0)
    h = ctx._h if ctx else None
    rc = lib().ig_partial_index(h, H, d, n, _ptr(Qs), _ptr(Ks), float(ratio), None, ctypes.byref(r))
    if rc != IG_OK:
        raise IgError(rc, ctx.last_error() if ctx else "ig_partial_index")
    idx = np.zeros((H, r.value), np.int32)
    rc = lib().ig_partial_index(h, H, d, n, _ptr(Qs), _ptr(Ks), float(ratio), _ptr(idx), ctypes.byref(r))
    if rc != IG_OK:
        raise IgError(rc, ctx.last_error() if ctx else "ig_partial_index")
    return idx


class Context:
    """Owns one ig_ctx.  Methods mirror the C entry points and raise IgError on a non-zero status."""

    def __init__(self, device: int = 0):
        h = _vp()
        rc = lib().ig_create(device, ctypes.byref(h))
        if rc != IG_OK:
            raise IgError(rc, "ig_create failed (no usable GPU?)")
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            lib().ig_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def last_error(self) -> str:
        return lib().ig_last_error(self._h).decode()

    def _ck(self, rc):
        if rc != IG_OK:
            raise IgError(rc, self.last_error())

    def call(self, name, *args):
        """Raw call returning the status code (used by error-path tests)."""
        return getattr(lib(), name)(self._h, *args)

    def ig_reserve(self, desc):
        self._ck(lib().ig_reserve(self._h, ctypes.byref(desc)))

    def ig_workspace_bytes(self) -> int:
        return int(lib().ig_workspace_bytes(self._h))

    def ig_check_status(self) -> int:
        return lib().ig_check_status(self._h)

    def ig_wq_build(self, desc, Wq, idx_dev, wq, stream=None):
        self._ck(lib().ig_wq_build(self._h, ctypes.byref(desc), _ptr(Wq), _ptr(idx_dev), _ptr(wq),
                                   _stream(stream)))

    def ig_slab_build(self, desc, Kpool, pool_space, idx_dev, slab, stream=None):
        self._ck(lib().ig_slab_build(self._h, ctypes.byref(desc), _ptr(Kpool), pool_space,
                                     _ptr(idx_dev), _ptr(slab), _stream(stream)))

    def ig_skew_device(self, D, H, n_cal, Qcal, A, sigma=None, stream=None):
        self._ck(lib().ig_skew_device(self._h, D, H, n_cal, _ptr(Qcal), _ptr(A), _ptr(sigma),
                                      _stream(stream)))

    def ig_partial_index_device(self, dtype, H, d, n, Qs, Ks, ratio, idx_dev, stream=None):
        self._ck(lib().ig_partial_index_device(self._h, dtype, H, d, n, _ptr(Qs), _ptr(Ks),
                                               float(ratio), _ptr(idx_dev), _stream(stream)))

    def ig_append_token(self, desc, k_new, v_new, idx_dev, slab, Kpool, Vpool, pool_space, stream=None):
        self._ck(lib().ig_append_token(self._h, ctypes.byref(desc), _ptr(k_new), _ptr(v_new),
                                       _ptr(idx_dev), _ptr(slab), _ptr(Kpool), _ptr(Vpool),
                                       pool_space, _stream(stream)))

    def ig_pool_touch(self, desc, sel_idx, sel_stride, sel_cnt, counters, counter_max=255, stream=None):
        self._ck(lib().ig_pool_touch(self._h, ctypes.byref(desc), _ptr(sel_idx), sel_stride,
                                     _ptr(sel_cnt), _ptr(counters), counter_max, _stream(stream)))

    def ig_pool_victim(self, desc, counters, victim, stream=None):
        self._ck(lib().ig_pool_victim(self._h, ctypes.byref(desc), _ptr(counters), _ptr(victim),
                                      _stream(stream)))

    def ig_pool_replace(self, desc, victim, k_new, v_new, idx_dev, slab, Kpool, Vpool, pool_space,
                        counters=None, stream=None):
        self._ck(lib().ig_pool_replace(self._h, ctypes.byref(desc), _ptr(victim), _ptr(k_new),
                                       _ptr(v_new), _ptr(idx_dev), _ptr(slab), _ptr(Kpool),
                                       _ptr(Vpool), pool_space, _ptr(counters), _stream(stream)))

    def ig_pool_touch_policy(self, desc, policy, sel_idx, sel_stride, sel_cnt, state, param, stream=None):
        self._ck(lib().ig_pool_touch_policy(self._h, ctypes.byref(desc), policy, _ptr(sel_idx), sel_stride,
                                            _ptr(sel_cnt), _ptr(state), param, _stream(stream)))

    def ig_pool_replace_policy(self, desc, policy, victim, k_new, v_new, idx_dev, slab, Kpool, Vpool,
                               pool_space, state, now, stream=None):
        self._ck(lib().ig_pool_replace_policy(self._h, ctypes.byref(desc), policy, _ptr(victim), _ptr(k_new),
                                              _ptr(v_new), _ptr(idx_dev), _ptr(slab), _ptr(Kpool),
                                              _ptr(Vpool), pool_space, _ptr(state), now, _stream(stream)))

    def ig_speculate(self, desc, x, wq, bias, A_p, pos, slab, sel_idx, sel_stride, sel_cnt,
                     scores_opt=None, stream=None):
        self._ck(lib().ig_speculate(self._h, ctypes.byref(desc), _ptr(x), _ptr(wq), _ptr(bias),
                                    _ptr(A_p), _ptr(pos), _ptr(slab), _ptr(sel_idx), sel_stride,
                                    _ptr(sel_cnt), _ptr(scores_opt), _stream(stream)))

    def ig_project(self, desc, x, wq, bias, A_p, pos, q_p, stream=None):
        self._ck(lib().ig_project(self._h, ctypes.byref(desc), _ptr(x), _ptr(wq), _ptr(bias),
                                  _ptr(A_p), _ptr(pos), _ptr(q_p), _stream(stream)))

    def ig_scan_select(self, desc, q_p, slab, sel_idx, sel_stride, sel_cnt, scores_opt=None,
                       stream=None):
        self._ck(lib().ig_scan_select(self._h, ctypes.byref(desc), _ptr(q_p), _ptr(slab),
                                      _ptr(sel_idx), sel_stride, _ptr(sel_cnt), _ptr(scores_opt),
                                      _stream(stream)))

    def ig_project_indexed(self, desc, x, Wq, idx_dev, bias, q_p, stream=None):
        self._ck(lib().ig_project_indexed(self._h, ctypes.byref(desc), _ptr(x), _ptr(Wq), _ptr(idx_dev),
                                          _ptr(bias), _ptr(q_p), _stream(stream)))

    def ig_speculate_indexed(self, desc, x, Wq, idx_dev, bias, slab, sel_idx, sel_stride, sel_cnt,
                             scores_opt=None, stream=None):
        self._ck(lib().ig_speculate_indexed(self._h, ctypes.byref(desc), _ptr(x), _ptr(Wq),
                                            _ptr(idx_dev), _ptr(bias), _ptr(slab), _ptr(sel_idx),
                                            sel_stride, _ptr(sel_cnt), _ptr(scores_opt),
                                            _stream(stream)))

    def ig_layer_step(self, desc, x, wq, bias, A_p, pos, slab, sel_idx_next, sel_cnt_next, q, Kpool,
                      Vpool, sel_idx, sel_cnt, sel_stride, K_sel, V_sel, k_new, v_new, out, stream=None):
        self._ck(lib().ig_layer_step(self._h, ctypes.byref(desc), _ptr(x), _ptr(wq), _ptr(bias),
                                     _ptr(A_p), _ptr(pos), _ptr(slab), _ptr(sel_idx_next),
                                     _ptr(sel_cnt_next), _ptr(q), _ptr(Kpool), _ptr(Vpool),
                                     _ptr(sel_idx), _ptr(sel_cnt), sel_stride, _ptr(K_sel), _ptr(V_sel),
                                     _ptr(k_new), _ptr(v_new), _ptr(out), _stream(stream)))

    def ig_gather_kv(self, desc, Kpool, Vpool, pool_space, sel_idx, sel_stride, sel_cnt, K_sel,
                     V_sel, stream=None):
        self._ck(lib().ig_gather_kv(self._h, ctypes.byref(desc), _ptr(Kpool), _ptr(Vpool),
                                    pool_space, _ptr(sel_idx), sel_stride, _ptr(sel_cnt),
                                    _ptr(K_sel), _ptr(V_sel), _stream(stream)))

    def ig_sparse_attention(self, desc, q, K_sel, V_sel, sel_cnt, sel_stride, k_new, v_new, out,
                            stream=None):
        self._ck(lib().ig_sparse_attention(self._h, ctypes.byref(desc), _ptr(q), _ptr(K_sel),
                                           _ptr(V_sel), _ptr(sel_cnt), sel_stride, _ptr(k_new),
                                           _ptr(v_new), _ptr(out), _stream(stream)))

    def ig_sparse_attention_static(self, desc, q, K_sel, V_sel, sel_cnt, sel_stride, k_new, v_new, out,
                                   stream=None):
        self._ck(lib().ig_sparse_attention_static(self._h, ctypes.byref(desc), _ptr(q), _ptr(K_sel),
                                                  _ptr(V_sel), _ptr(sel_cnt), sel_stride, _ptr(k_new),
                                                  _ptr(v_new), _ptr(out), _stream(stream)))

    def ig_sparse_attention_indexed(self, desc, q, Kpool, Vpool, sel_idx, sel_stride, sel_cnt,
                                    k_new, v_new, out, stream=None):
        self._ck(lib().ig_sparse_attention_indexed(self._h, ctypes.byref(desc), _ptr(q),
                                                   _ptr(Kpool), _ptr(Vpool), _ptr(sel_idx),
                                                   sel_stride, _ptr(sel_cnt), _ptr(k_new),
                                                   _ptr(v_new), _ptr(out), _stream(stream)))

    def ig_speculate_equalized(self, desc, x, wq, bias, A_p, pos, slab, max_frac, sel_idx, sel_stride, sel_cnt,
                               thr_cnt_opt=None, stream=None):
        self._ck(self.call("ig_speculate_equalized", ctypes.byref(desc), _ptr(x), _ptr(wq), _ptr(bias), _ptr(A_p),
                           _ptr(pos), _ptr(slab), float(max_frac), _ptr(sel_idx), sel_stride, _ptr(sel_cnt),
                           _ptr(thr_cnt_opt), _stream(stream)))

    def ig_equalize_heads(self, desc, scores, thr_cnt, max_frac, sel_idx, sel_stride, sel_cnt,
                          stream=None):
        self._ck(lib().ig_equalize_heads(self._h, ctypes.byref(desc), _ptr(scores), _ptr(thr_cnt),
                                         float(max_frac), _ptr(sel_idx), sel_stride, _ptr(sel_cnt),
                                         _stream(stream)))

    def ig_gather_attention(self, desc, q, Kpool, Vpool, sel_idx, sel_stride, sel_cnt, K_sel, V_sel,
                            k_new, v_new, out, stream=None):
        self._ck(lib().ig_gather_attention(self._h, ctypes.byref(desc), _ptr(q), _ptr(Kpool),
                                           _ptr(Vpool), _ptr(sel_idx), sel_stride, _ptr(sel_cnt),
                                           _ptr(K_sel), _ptr(V_sel), _ptr(k_new), _ptr(v_new),
                                           _ptr(out), _stream(stream)))

    def ig_decode_step_overlapped(self, desc, layers, wq, bias, A_p, pos, pool_space, sets, sel_stride,
                                  main_stream, side_stream):
        """layers: ctypes array of IgLayerIO; sets: ctypes array of IgBufferSet (kept by the caller)."""
        self._ck(self.call("ig_decode_step_overlapped", ctypes.byref(desc), len(layers), ctypes.addressof(layers),
                           _ptr(wq), _ptr(bias), _ptr(A_p), _ptr(pos), pool_space, len(sets), ctypes.addressof(sets),
                           sel_stride, _stream(main_stream), _stream(side_stream)))

    def ig_set_wait_limit(self, ticks: int):
        self._ck(lib().ig_set_wait_limit(self._h, int(ticks)))

    def ig_profile_begin(self):
        self._ck(lib().ig_profile_begin(self._h))

    def ig_profile_end(self):
        self._ck(lib().ig_profile_end(self._h))

    def ig_profile_read(self, which):
        ms, n = ctypes.c_double(0), _i32(0)
        self._ck(lib().ig_profile_read(self._h, which, ctypes.byref(ms), ctypes.byref(n)))
        return ms.value, n.value

    def ig_copy_bytes(self, src, dst, nbytes, stream=None):
        self._ck(lib().ig_copy_bytes(self._h, _ptr(src), _ptr(dst), nbytes, _stream(stream)))

    def ig_read_bytes(self, src, nbytes, stream=None):
        self._ck(lib().ig_read_bytes(self._h, _ptr(src), nbytes, _stream(stream)))
