"""GPU parity of the head-equalised selection (ig_equalize_heads) against the CPU oracle.

The selection is integer work on float32 scores, so on identical scores the lists must be
bit-exact.  End to end (GPU scores against oracle scores, which differ by summation order) a token
may differ only if its oracle score lies within 1e-3 of the oracle's n-th largest score."""
import numpy as np
import pytest
import torch

import ig_workloads as wl
from ig_case import make_case, run_oracle
from oracle import ig_oracle as o

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_2406_19707_amd as ig
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = ig.Context(0)
    yield c
    c.close()


def equalize_on_gpu(ctx, scores, thr_cnt, alpha, max_frac, stride=None):
    import paper_2406_19707_amd as ig
    B, H, N = scores.shape
    stride = N if stride is None else stride
    d = ig.IgDesc(B=B, H=H, d=64, r=8, N=N, alpha=alpha)
    s_dev = torch.from_numpy(np.ascontiguousarray(scores)).cuda()
    c_dev = torch.from_numpy(np.ascontiguousarray(thr_cnt.astype(np.int32))).cuda()
    idx = torch.full((B * H, stride), -1, dtype=torch.int32, device="cuda")
    cnt = torch.full((B * H,), -1, dtype=torch.int32, device="cuda")
    ctx.ig_equalize_heads(d, s_dev, c_dev, max_frac, idx, stride, cnt)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), cnt.cpu().numpy(), ctx.ig_check_status()


def assert_same_lists(idx, cnt, ref_idx, ref_cnt):
    assert np.array_equal(cnt, ref_cnt)
    for i in range(len(cnt)):
        assert np.array_equal(idx[i, :cnt[i]], ref_idx[i, :cnt[i]]), i


@pytest.mark.parametrize("B,H,N,alpha,max_frac,ties", [
    (2, 4, 2048, 4.0, 0.2, False),
    (3, 5, 1999, 2.0, 0.2, True),      # ragged length, many equal scores
    (1, 3, 257, 1.0, 1.0, True),
    (2, 2, 5, 0.0, 0.2, True),         # cap floors to 1
    (1, 2, 20000, 3.0, 0.2, False),    # long sequence: 1024-thread workgroups
    (1, 2, 9000, 3.0, 0.5, True),
    (4, 40, 700, 3.0, 0.2, False),     # more heads than a wave
])
def test_bit_exact_on_given_scores(ctx, B, H, N, alpha, max_frac, ties):
    print(f"case B{B} H{H} N{N} alpha {alpha} max_frac {max_frac} ties {ties}", flush=True)
    rng = np.random.default_rng(B * 1000 + H * 100 + N)
    s = (rng.standard_normal((B, H, N)) * rng.uniform(0.5, 3.0, (B, H, 1))).astype(np.float32)
    if ties:
        s = (np.round(s * 2) / 2).astype(np.float32)
        s[0, 0, ::3] = -0.0            # signed zeros compare equal
        s[0, 0, 1::3] = 0.0
    _, thr_cnt = o.select(s, alpha)
    ref_idx, ref_cnt, _ = o.select_equalized(s, alpha, max_frac)
    idx, cnt, status = equalize_on_gpu(ctx, s, thr_cnt, alpha, max_frac)
    assert status == 0
    assert_same_lists(idx, cnt, ref_idx, ref_cnt)


def test_all_scores_equal_keeps_the_earliest_tokens_up_to_the_cap(ctx):
    s = np.zeros((1, 2, 2048), np.float32)
    idx, cnt, status = equalize_on_gpu(ctx, s, np.full(2, 2048), 4.0, 0.2)
    assert status == 0 and np.all(cnt == 409)
    assert np.array_equal(idx[:, :409], np.tile(np.arange(409, dtype=np.int32), (2, 1)))


def test_short_stride_is_clamped_and_flagged(ctx):
    import paper_2406_19707_amd as ig
    s = np.random.default_rng(1).standard_normal((1, 2, 512)).astype(np.float32)
    ref_idx, _, _ = o.select_equalized(s, 100.0, 1.0)          # everything kept
    idx, cnt, status = equalize_on_gpu(ctx, s, np.full(2, 512), 100.0, 1.0, stride=100)
    assert status == ig.IG_ECAPACITY and np.all(cnt == 100)
    assert np.array_equal(idx, ref_idx[:, :100])


def test_error_paths(ctx):
    import ctypes
    import paper_2406_19707_amd as ig
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    p = buf.data_ptr()
    d = ig.IgDesc(B=1, H=2, d=128, r=38, N=64)
    call = lambda frac, cnt_out=p + 4096: ctx.call(  # noqa: E731
        "ig_equalize_heads", ctypes.byref(d), p, p + 2048, ctypes.c_double(frac), p + 8192, 64, cnt_out, 0)
    assert call(0.0) == ig.IG_EINVAL
    assert call(1.5) == ig.IG_EINVAL
    assert call(float("nan")) == ig.IG_EINVAL
    assert call(0.2, cnt_out=p + 2048) == ig.IG_EINVAL and "alias" in ctx.last_error()


@pytest.mark.parametrize("cfg,shape,gain", [
    (2, dict(B=3, H=4, N=2048), 6.0),
    (3, dict(B=2, H=4, N=4096), 24.0),
    (5, dict(B=1, H=2, N=20000), 6.0),
])
def test_end_to_end_with_speculated_scores(ctx, cfg, shape, gain):
    """ig_speculate (scores + threshold counts) -> ig_equalize_heads -> gather -> attention."""
    import paper_2406_19707_amd as ig
    from ig_gpu import Uploaded
    w = wl.shrink(wl.WORKLOADS[cfg], **shape, pool="hbm")
    c = make_case(w, gain=gain)
    print(f"case {w.name} B{w.B} H{w.H} N{c.N}", flush=True)
    ref = run_oracle(c)
    up = Uploaded(ctx, c)
    d = up.desc
    BH, N = w.B * w.H, c.N
    tdt = torch.float16
    scores = torch.zeros((w.B, w.H, N), device="cuda")
    t_idx = torch.zeros((BH, N), dtype=torch.int32, device="cuda")
    t_cnt = torch.zeros((BH,), dtype=torch.int32, device="cuda")
    e_idx = torch.full((BH, N), -1, dtype=torch.int32, device="cuda")
    e_cnt = torch.zeros((BH,), dtype=torch.int32, device="cuda")
    K_sel = torch.zeros((BH, N, w.d), dtype=tdt, device="cuda")
    V_sel = torch.zeros_like(K_sel)
    out = torch.zeros((w.B, w.H, w.d), dtype=tdt, device="cuda")
    # (1) equalisation fed with the oracle's scores and threshold counts (inputs flow oracle -> HIP
    # path): integer work on identical floats, so the lists are bit-exact
    r_idx, r_cnt, r_n = o.select_equalized(ref.s, w.alpha, 0.2)
    ctx.ig_equalize_heads(d, torch.from_numpy(ref.s).cuda(), torch.from_numpy(ref.sel_cnt).cuda(), 0.2,
                          e_idx, N, e_cnt)
    torch.cuda.synchronize()
    assert_same_lists(e_idx.cpu().numpy(), e_cnt.cpu().numpy(), r_idx, r_cnt)
    # (2) rows and attention over the oracle's equalised lists
    ctx.ig_gather_kv(d, up.K, up.V, ig.IG_MEM_DEVICE, e_idx, N, e_cnt, K_sel, V_sel)
    ctx.ig_sparse_attention(d, up.q, K_sel, V_sel, e_cnt, N, None, None, out)
    torch.cuda.synchronize()
    Ks = o.gather(c.f32("Kt"), r_idx, r_cnt)
    Vs = o.gather(c.f32("V"), r_idx, r_cnt)
    n_max = int(r_cnt.max())
    assert np.array_equal(K_sel.float().cpu().numpy()[:, :n_max], Ks[:, :n_max])
    assert np.array_equal(V_sel.float().cpu().numpy()[:, :n_max], Vs[:, :n_max])
    ref_out = o.attend(c.f32("q"), Ks, Vs, r_cnt, c.scale)
    err = np.abs(out.float().cpu().numpy().reshape(BH, w.d) - ref_out)
    assert np.all(err <= 2e-2 + 1e-2 * np.abs(ref_out)), err.max()
    # (3) the whole chain on the GPU (its own scores, which differ from the oracle's by summation
    # order): the per-sequence count may move by the tokens inside the 1e-3 band of a threshold,
    # and with equal counts only tokens within 1e-3 of the oracle's n-th largest score may differ
    ctx.ig_speculate(d, up.x, up.wq, up.bias, up.A_p, up.pos, up.slab, t_idx, N, t_cnt, scores)
    ctx.ig_equalize_heads(d, scores, t_cnt, 0.2, e_idx, N, e_cnt)
    torch.cuda.synchronize()
    assert ctx.ig_check_status() == 0
    g_idx, g_cnt = e_idx.cpu().numpy(), e_cnt.cpu().numpy()
    assert np.all(np.abs(g_cnt - r_cnt) <= 1)
    s2 = ref.s.reshape(BH, N)
    for i in range(BH):
        assert np.all(np.diff(g_idx[i, :g_cnt[i]]) > 0)
        if g_cnt[i] != r_cnt[i]:
            continue
        diff = np.setxor1d(g_idx[i, :g_cnt[i]], r_idx[i, :r_cnt[i]])
        if diff.size:
            nth = np.sort(s2[i])[::-1][r_cnt[i] - 1]
            assert np.all(np.abs(s2[i, diff] - nth) <= 1e-3)
    print(f"  equalised count per sequence {r_n}, mean threshold count {ref.sel_cnt.mean():.1f}", flush=True)


# ---- ig_speculate_equalized: the selection inside the scan kernel ---------------------------------

def two_kernel_reference(ctx, up, N, max_frac):
    d = up.desc
    w = up.c.w
    BH = w.B * w.H
    scores = torch.zeros((w.B, w.H, N), device="cuda")
    t_idx = torch.zeros((BH, N), dtype=torch.int32, device="cuda")
    t_cnt = torch.zeros((BH,), dtype=torch.int32, device="cuda")
    e_idx = torch.full((BH, N), -1, dtype=torch.int32, device="cuda")
    e_cnt = torch.zeros((BH,), dtype=torch.int32, device="cuda")
    ctx.ig_speculate(d, up.x, up.wq, up.bias, up.A_p, up.pos, up.slab, t_idx, N, t_cnt, scores)
    ctx.ig_equalize_heads(d, scores, t_cnt, max_frac, e_idx, N, e_cnt)
    torch.cuda.synchronize()
    return scores.cpu().numpy(), t_cnt.cpu().numpy(), e_idx.cpu().numpy(), e_cnt.cpu().numpy()


@pytest.mark.parametrize("cfg,shape,gain,max_frac,fused", [
    (2, dict(B=4, H=32, N=2048), 20.0, 0.2, True),     # one tile per wave
    (2, dict(B=5, H=32, N=1800), 32.0, 0.05, True),    # ragged last tile, the cap binds
    (3, dict(B=4, H=32, N=4096), 40.0, 0.2, True),     # rotary prologue, two tiles per wave
    (3, dict(B=3, H=48, N=3000), 30.0, 0.2, True),     # ragged, H not a multiple of 8
    (2, dict(B=2, H=40, N=300), 12.0, 1.0, False),     # too few pairs for the streaming form: two kernels
    (5, dict(B=1, H=8, N=20000), 6.0, 0.2, False),     # long sequence: two kernels
])
def test_speculate_equalized_matches_the_two_calls_and_the_oracle(cfg, shape, gain, max_frac, fused):
    import paper_2406_19707_amd as ig
    from ig_gpu import Uploaded
    ctx = ig.Context(0)
    w = wl.shrink(wl.WORKLOADS[cfg], **shape, pool="hbm", n_cal=256)
    c = make_case(w, gain=gain)
    print(f"case {w.name} B{w.B} H{w.H} N{c.N} r{c.r} rope={w.rope} max_frac={max_frac}", flush=True)
    up = Uploaded(ctx, c)
    d = up.desc
    BH, N = w.B * w.H, c.N
    scores, t_cnt, ref_idx, ref_cnt = two_kernel_reference(ctx, up, N, max_frac)
    # the reference itself against the oracle on the GPU's scores (exact) ...
    o_idx, o_cnt, _ = o.select_equalized(scores, w.alpha, max_frac)
    assert_same_lists(ref_idx, ref_cnt, o_idx, o_cnt)
    assert 0 < ref_cnt.min() and ref_cnt.max() < N
    for limit, what in ((None, "waits"), (-1, "every workgroup alone"), (None, "waits again")):
        if limit is not None:
            ctx.ig_set_wait_limit(limit)
        idx = torch.full((BH, N), -1, dtype=torch.int32, device="cuda")
        cnt = torch.full((BH,), -1, dtype=torch.int32, device="cuda")
        thr = torch.full((BH,), -1, dtype=torch.int32, device="cuda")
        ctx.ig_speculate_equalized(d, up.x, up.wq, up.bias, up.A_p, up.pos, up.slab, max_frac, idx, N, cnt, thr)
        torch.cuda.synchronize()
        assert ctx.ig_check_status() == ig.IG_OK, what
        assert np.array_equal(thr.cpu().numpy(), t_cnt), what
        assert_same_lists(idx.cpu().numpy(), cnt.cpu().numpy(), ref_idx, ref_cnt)
        if limit is not None:
            ctx.ig_set_wait_limit(2000000)
    # without the optional counts; the kernels launched tell which route the shape took
    idx = torch.full((BH, N), -1, dtype=torch.int32, device="cuda")
    cnt = torch.full((BH,), -1, dtype=torch.int32, device="cuda")
    ctx.ig_profile_begin()
    ctx.ig_speculate_equalized(d, up.x, up.wq, up.bias, up.A_p, up.pos, up.slab, max_frac, idx, N, cnt)
    torch.cuda.synchronize()
    ctx.ig_profile_end()
    assert_same_lists(idx.cpu().numpy(), cnt.cpu().numpy(), ref_idx, ref_cnt)
    assert ctx.ig_profile_read(ig.IG_K_SCAN)[1] >= 1
    assert (ctx.ig_profile_read(ig.IG_K_SELECT)[1] == 0) == fused, "route taken is not the one this case is for"
    # a short stride is clamped and flagged
    if fused:
        short = int(ref_cnt.max()) - 1
        idx = torch.full((BH, short), -1, dtype=torch.int32, device="cuda")
        ctx.ig_speculate_equalized(d, up.x, up.wq, up.bias, up.A_p, up.pos, up.slab, max_frac, idx, short, cnt)
        torch.cuda.synchronize()
        assert ctx.ig_check_status() == ig.IG_ECAPACITY
        got = idx.cpu().numpy()
        for i in range(BH):
            k = min(short, int(ref_cnt[i]))
            assert np.array_equal(got[i, :k], ref_idx[i, :k])
    ctx.close()


def test_speculate_equalized_error_paths(ctx):
    import ctypes
    import paper_2406_19707_amd as ig
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    p = buf.data_ptr()
    d = ig.IgDesc(B=1, H=2, d=128, r=38, N=64)
    def call(frac, slab=p + 4096, cnt=p + 65536, thr=0):
        return ctx.call("ig_speculate_equalized", ctypes.byref(d), p, p + 1024, 0, 0, 0, slab,
                        ctypes.c_double(frac), p + 131072, 64, cnt, thr, 0)
    assert call(0.0) == ig.IG_EINVAL
    assert call(1.5) == ig.IG_EINVAL
    assert call(float("nan")) == ig.IG_EINVAL
    assert call(0.2, slab=0) == ig.IG_EINVAL
    assert call(0.2, cnt=0) == ig.IG_EINVAL
    assert call(0.2, cnt=p + 65536, thr=p + 65536) == ig.IG_EINVAL and "alias" in ctx.last_error()
