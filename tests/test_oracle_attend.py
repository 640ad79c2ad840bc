"""Pins for the oracle's gather and sparse decode attention (Sections 2.1, 4.1, 4.3) and for the
whole oracle pipeline's limiting cases."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import ig_workloads as wl
from oracle import ig_oracle as o


def dense_attention_torch(q, K, V, scale, mask=None):
    """Library routine: torch's scaled_dot_product_attention in float64 on the CPU."""
    qt = torch.from_numpy(q.astype(np.float64))[:, None, :]           # [BH, 1, d]
    Kt = torch.from_numpy(K.astype(np.float64))
    Vt = torch.from_numpy(V.astype(np.float64))
    m = None if mask is None else torch.from_numpy(mask)[:, None, :]
    return F.scaled_dot_product_attention(qt, Kt, Vt, attn_mask=m, scale=scale)[:, 0, :].numpy()


def test_gather_is_a_row_copy():
    rng = np.random.default_rng(0)
    BH, N, d = 5, 33, 6
    pool = rng.standard_normal((BH, N, d)).astype(np.float32)
    cnt = np.array([0, 1, 33, 7, 12], np.int32)
    idx = np.full((BH, N), -1, np.int32)
    for i in range(BH):
        idx[i, :cnt[i]] = np.sort(rng.choice(N, cnt[i], replace=False))
    out = o.gather(pool, idx, cnt)
    for i in range(BH):
        assert np.array_equal(out[i, :cnt[i]], pool[i, idx[i, :cnt[i]]])
        assert np.all(out[i, cnt[i]:] == 0)


def test_attend_over_all_rows_is_dense_attention():
    rng = np.random.default_rng(1)
    BH, N, d, scale = 6, 50, 16, 0.25
    q = rng.standard_normal((BH, d)).astype(np.float32)
    K = rng.standard_normal((BH, N, d)).astype(np.float32)
    V = rng.standard_normal((BH, N, d)).astype(np.float32)
    cnt = np.full(BH, N, np.int32)
    got = o.attend(q, K, V, cnt, scale)
    assert np.abs(got - dense_attention_torch(q, K, V, scale)).max() <= 1e-6


def test_attend_on_selected_rows_is_masked_dense_attention():
    rng = np.random.default_rng(2)
    BH, N, d, scale = 4, 40, 8, 0.5
    q = rng.standard_normal((BH, d)).astype(np.float32)
    K = rng.standard_normal((BH, N, d)).astype(np.float32)
    V = rng.standard_normal((BH, N, d)).astype(np.float32)
    cnt = np.array([1, 5, 17, 40], np.int32)
    idx = np.full((BH, N), -1, np.int32)
    mask = np.zeros((BH, N), bool)
    for i in range(BH):
        idx[i, :cnt[i]] = np.sort(rng.choice(N, cnt[i], replace=False))
        mask[i, idx[i, :cnt[i]]] = True
    got = o.attend(q, o.gather(K, idx, cnt), o.gather(V, idx, cnt), cnt, scale)
    assert np.abs(got - dense_attention_torch(q, K, V, scale, mask)).max() <= 1e-6


def test_attend_weights_sum_to_one_and_output_is_convex():
    rng = np.random.default_rng(3)
    BH, n, d = 3, 9, 4
    q = rng.standard_normal((BH, d)).astype(np.float32) * 3
    K = rng.standard_normal((BH, n, d)).astype(np.float32)
    V = rng.standard_normal((BH, n, d)).astype(np.float32)
    cnt = np.array([9, 4, 1], np.int32)
    ones = o.attend(q, K, np.ones_like(V), cnt, 1.0)
    assert np.allclose(ones, 1.0, atol=1e-6)
    out = o.attend(q, K, V, cnt, 1.0)
    for i in range(BH):
        assert np.all(out[i] <= V[i, :cnt[i]].max(0) + 1e-6)
        assert np.all(out[i] >= V[i, :cnt[i]].min(0) - 1e-6)
    assert np.allclose(out[2], V[2, 0], atol=1e-6)            # a single row gets weight 1


def test_attend_is_shift_invariant_and_stable_for_large_logits():
    q = np.array([[100.0, 0.0]], np.float32)
    K = np.array([[[10.0, 0], [9.0, 0], [0, 5.0]]], np.float32)
    V = np.array([[[1.0, 0], [0, 1.0], [7, 7]]], np.float32)
    out = o.attend(q, K, V, np.array([3], np.int32), 1.0)     # logits 1000, 900, 0
    assert np.all(np.isfinite(out)) and np.allclose(out[0], [1.0, 0.0], atol=1e-6)


def test_new_token_row_is_always_attended():
    rng = np.random.default_rng(4)
    BH, n, d, scale = 3, 6, 8, 0.3
    q = rng.standard_normal((BH, d)).astype(np.float32)
    K = rng.standard_normal((BH, n, d)).astype(np.float32)
    V = rng.standard_normal((BH, n, d)).astype(np.float32)
    kn = rng.standard_normal((BH, d)).astype(np.float32)
    vn = rng.standard_normal((BH, d)).astype(np.float32)
    cnt = np.array([6, 2, 0], np.int32)
    got = o.attend(q, K, V, cnt, scale, kn, vn)
    for i in range(BH):
        Kc = np.concatenate([K[i, :cnt[i]], kn[i:i + 1]])[None]
        Vc = np.concatenate([V[i, :cnt[i]], vn[i:i + 1]])[None]
        assert np.abs(got[i] - dense_attention_torch(q[i:i + 1], Kc, Vc, scale)[0]).max() <= 1e-6


@pytest.mark.parametrize("rope", [False, True])
def test_pipeline_with_all_columns_and_infinite_alpha_is_dense_attention(rope):
    # spec limiting case: idx = every column and alpha = inf -> the whole path reproduces
    # dense attention with the unskewed weights on the layer's own input.
    w = wl.shrink(wl.WORKLOADS[1], B=2, N=96, n_cal=128, rope=rope)
    Wq, Wk = wl.projection_weight(w, "Wq"), wl.projection_weight(w, "Wk")
    Xcal = wl.calibration_input(w)
    K, V = wl.kv_cache(w)                                       # K = un-skewed keys [B,H,N,d]
    x = wl.attention_input(w)
    pos_cal = np.arange(w.n_cal, dtype=np.int32)
    pos = np.full(w.B, w.N, np.int32)
    Qcal = (Xcal @ Wq)
    if rope:
        Qcal = o.rope(Qcal.reshape(w.n_cal, w.H, w.d), pos_cal).reshape(w.n_cal, w.D)
    sk = o.skew(Wq, Wk, Qcal, w.H)
    idx = np.tile(np.arange(w.d, dtype=np.int32), (w.H, 1))
    Kt = o.apply_skew(K.transpose(0, 2, 1, 3), sk["A"]).transpose(0, 2, 1, 3)
    scale = 1.0 / np.sqrt(w.d)
    if rope:
        qp = o.project_rope(x, Wq, pos, sk["A"], idx)
        q_plain = o.rope((x @ Wq).reshape(w.B, w.H, w.d), pos)
    else:
        qp = o.project(x, sk["Wq_s"], idx)
        q_plain = (x @ Wq).reshape(w.B, w.H, w.d)
    s = o.scan(qp, Kt, idx, scale)
    sel_idx, sel_cnt = o.select(s, np.inf)
    assert np.all(sel_cnt == w.N)
    out = o.attend(qp, o.gather(Kt, sel_idx, sel_cnt), o.gather(V, sel_idx, sel_cnt), sel_cnt, scale)
    ref = dense_attention_torch(q_plain.reshape(-1, w.d), K.reshape(-1, w.N, w.d),
                                V.reshape(-1, w.N, w.d), scale)
    assert np.abs(out - ref).max() <= 1e-5 * max(1.0, np.abs(ref).max())
    # and the speculated scores are the true logits
    ref_s = scale * np.einsum("bhd,bhnd->bhn", q_plain.astype(np.float64), K.astype(np.float64))
    assert np.abs(s - ref_s).max() <= 1e-5 * np.abs(ref_s).max() + 1e-6
