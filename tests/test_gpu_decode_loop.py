"""GPU parity of the growing cache: ig_append_token, then the hot path on the longer cache, several
decode steps in a row (Section 2.1: the key and value of each generated token join the cache;
Section 4.4: the partial key cache is updated with them).  The oracle sees the same cache as plain
arrays cut to the current length."""
import numpy as np
import pytest
import torch

import ig_workloads as wl
from ig_case import make_case, compare_selection, OracleResult
from oracle import ig_oracle as o

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_2406_19707_amd as ig
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = ig.Context(0)
    yield c
    c.close()


def oracle_at_length(c, n):
    w = c.w
    if w.rope:
        q_p = o.project_rope(c.f32("x"), c.f32("W_in"), c.pos, c.A, c.idx)
    else:
        q_p = o.project(c.f32("x"), c.f32("W_in"), c.idx)
    Kt = c.f32("Kt")
    s = o.scan(q_p, Kt, c.idx, c.scale, N=n)
    sel_idx, sel_cnt = o.select(s, w.alpha)
    K_sel = o.gather(Kt, sel_idx, sel_cnt)
    V_sel = o.gather(c.f32("V"), sel_idx, sel_cnt)
    out = o.attend(c.f32("q"), K_sel, V_sel, sel_cnt, c.scale)
    return OracleResult(q_p, s, sel_idx, sel_cnt, K_sel, V_sel, out, None)


@pytest.mark.parametrize("cfg,shape,gain,N0,T,host_pool", [
    (2, dict(B=2, H=4), 6.0, 1020, 8, False),      # crosses the 512-token tile boundary at 1024
    (3, dict(B=2, H=2), 16.0, 509, 6, False),      # rope, crosses 512
    (4, dict(B=3, H=2), 6.0, 700, 4, True),        # pinned host pool: rows are written over PCIe
    (1, dict(), 8.0, 250, 10, False),              # float32: 256-token tiles
    (2, dict(B=1, H=2), 6.0, 0, 5, False),         # from an empty cache
])
def test_append_then_hot_path_over_several_steps(ctx, cfg, shape, gain, N0, T, host_pool):
    import paper_2406_19707_amd as ig
    from ig_gpu import desc_of, dev
    w = wl.shrink(wl.WORKLOADS[cfg], N=N0 + T, heavy_count=min(8, N0 + T), pool="hbm", **shape)
    c = make_case(w, gain=gain)
    print(f"case {w.name} B{w.B} H{w.H} N0 {N0} steps {T} host_pool {host_pool}", flush=True)
    N_cap = N0 + T
    tdt = torch.float32 if w.dtype == "f32" else torch.float16
    BH = w.B * w.H
    # pools hold the first N0 tokens; the slots behind them hold junk until they are appended
    Kh, Vh = c.Kt.copy(), c.V.copy()
    Kh[:, :, N0:] = 9.0
    Vh[:, :, N0:] = -9.0
    if host_pool:
        K, V, space = torch.from_numpy(Kh).pin_memory(), torch.from_numpy(Vh).pin_memory(), ig.IG_MEM_HOST_PINNED
    else:
        K, V, space = dev(Kh), dev(Vh), ig.IG_MEM_DEVICE
    d = desc_of(c, N=max(N0, 1))
    d.N_cap = N_cap
    x, W, idx, q = dev(c.x), dev(c.W_in), dev(c.idx), dev(c.q)
    A_p = dev(c.A_p) if w.rope else None
    pos = dev(c.pos) if w.rope else None
    wq = torch.empty(ig.ig_wq_bytes(d), dtype=torch.uint8, device="cuda")
    slab = torch.empty(ig.ig_slab_bytes(d), dtype=torch.uint8, device="cuda")
    ctx.ig_wq_build(d, W, idx, wq)
    if N0 > 0:
        ctx.ig_slab_build(d, K, space, idx, slab)
    else:
        slab.zero_()
    sel_idx = torch.zeros((BH, N_cap), dtype=torch.int32, device="cuda")
    sel_cnt = torch.zeros((BH,), dtype=torch.int32, device="cuda")
    K_sel = torch.zeros((BH, N_cap, w.d), dtype=tdt, device="cuda")
    V_sel = torch.zeros_like(K_sel)
    out = torch.zeros((w.B, w.H, w.d), dtype=tdt, device="cuda")
    Kfull, Vfull = dev(c.Kt), dev(c.V)
    for i in range(T):
        n = N0 + i
        d.N = n                                          # the cache before the append
        k_new = Kfull[:, :, n].contiguous()
        v_new = Vfull[:, :, n].contiguous()
        ctx.ig_append_token(d, k_new, v_new, idx, slab, K, V, space)
        d.N = n + 1
        ctx.ig_speculate(d, x, wq, None, A_p, pos, slab, sel_idx, N_cap, sel_cnt, None)
        ctx.ig_gather_kv(d, K, V, space, sel_idx, N_cap, sel_cnt, K_sel, V_sel)
        ctx.ig_sparse_attention(d, q, K_sel, V_sel, sel_cnt, N_cap, None, None, out)
        torch.cuda.synchronize()
        assert ctx.ig_check_status() == 0
        ref = oracle_at_length(c, n + 1)
        g_idx, g_cnt = sel_idx.cpu().numpy(), sel_cnt.cpu().numpy()
        slack = compare_selection(g_idx, g_cnt, ref, w.alpha)
        Kt3, V3 = c.Kt.reshape(BH, N_cap, w.d), c.V.reshape(BH, N_cap, w.d)
        Ks, Vs = K_sel.cpu().numpy(), V_sel.cpu().numpy()
        for j in range(BH):
            rows = g_idx[j, :g_cnt[j]]
            assert np.array_equal(Ks[j, :g_cnt[j]], Kt3[j, rows]) and np.array_equal(Vs[j, :g_cnt[j]], V3[j, rows])
        if slack == 0:
            atol, rtol = (1e-4, 1e-4) if w.dtype == "f32" else (2e-2, 1e-2)
            err = np.abs(out.float().cpu().numpy().reshape(BH, w.d) - ref.out)
            assert np.all(err <= atol + rtol * np.abs(ref.out)), (i, err.max())
    # the pools now hold exactly the full cache
    assert np.array_equal(K.cpu().numpy(), c.Kt) and np.array_equal(V.cpu().numpy(), c.V)


def test_append_to_a_full_cache_is_refused(ctx):
    import ctypes
    import paper_2406_19707_amd as ig
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    p = buf.data_ptr()
    d = ig.IgDesc(B=1, H=2, d=128, r=38, N=64, N_cap=64)
    rc = ctx.call("ig_append_token", ctypes.byref(d), p, p, p, p, p, p, ig.IG_MEM_DEVICE, 0)
    assert rc == ig.IG_ECAPACITY and "full" in ctx.last_error()
    d = ig.IgDesc(B=1, H=2, d=128, r=38, N=10, N_cap=64)
    assert ctx.call("ig_append_token", ctypes.byref(d), None, p, p, p, p, p, ig.IG_MEM_DEVICE, 0) == ig.IG_EINVAL
    assert ctx.call("ig_append_token", ctypes.byref(d), p + 8, p, p, p, p, p, ig.IG_MEM_DEVICE, 0) == ig.IG_EINVAL
