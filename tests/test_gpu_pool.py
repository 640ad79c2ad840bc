"""GPU parity of the counter-based KV pool management (Section 4.4) against the CPU oracle:
counters and victims bit-exact; a full cache that keeps decoding (victim overwritten by the new
token in the pool and in the partial key cache) checked step by step."""
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


@pytest.mark.parametrize("BH,N,N_cap,cmax,seed", [(8, 2048, 2048, 255, 1), (6, 700, 1024, 4, 2),
                                                  (3, 5, 8, 2, 3), (4, 20000, 20000, 7, 4)])
def test_counters_and_victims_are_bit_exact(ctx, BH, N, N_cap, cmax, seed):
    import paper_2406_19707_amd as ig
    print(f"case BH{BH} N{N}/{N_cap} counter_max {cmax}", flush=True)
    rng = np.random.default_rng(seed)
    d = ig.IgDesc(B=1, H=BH, d=64, r=8, N=N, N_cap=N_cap)
    counters = rng.integers(0, cmax, (BH, N_cap)).astype(np.int32)
    c_dev = torch.from_numpy(counters.copy()).cuda()
    victim = torch.full((BH,), -1, dtype=torch.int32, device="cuda")
    for step in range(4):
        idx = np.full((BH, N_cap), -1, np.int32)
        cnt = np.zeros(BH, np.int32)
        for i in range(BH):
            n = int(rng.integers(0, max(2, N // 4)))
            if step == 3 and i == 0:
                n = 0                                      # an empty list changes nothing
            idx[i, :n] = np.sort(rng.choice(N, n, replace=False))
            cnt[i] = n
        o.pool_touch(counters, idx, cnt, N, counter_max=cmax)
        ctx.ig_pool_touch(d, torch.from_numpy(idx).cuda(), N_cap, torch.from_numpy(cnt).cuda(), c_dev, cmax)
        ctx.ig_pool_victim(d, c_dev, victim)
        torch.cuda.synchronize()
        assert np.array_equal(c_dev.cpu().numpy(), counters), step
        assert np.array_equal(victim.cpu().numpy(), o.pool_victim(counters, N)), step


@pytest.mark.parametrize("cfg,shape,gain,N,T,host_pool", [
    (2, dict(B=2, H=4), 6.0, 1024, 6, False),
    (3, dict(B=2, H=2), 16.0, 700, 5, False),
    (4, dict(B=2, H=2), 6.0, 600, 4, True),
])
def test_full_cache_keeps_decoding_with_eviction(ctx, cfg, shape, gain, N, T, host_pool):
    import paper_2406_19707_amd as ig
    from ig_gpu import desc_of, dev
    w = wl.shrink(wl.WORKLOADS[cfg], N=N, heavy_count=8, pool="hbm", **shape)
    c = make_case(w, gain=gain)
    print(f"case {w.name} B{w.B} H{w.H} N{N} steps {T} host_pool {host_pool}", flush=True)
    BH = w.B * w.H
    tdt = torch.float16
    rng = np.random.default_rng(99)
    Kh, Vh = c.Kt.copy(), c.V.copy()                       # host mirror of the pools
    if host_pool:
        K, V, space = torch.from_numpy(Kh.copy()).pin_memory(), torch.from_numpy(Vh.copy()).pin_memory(), ig.IG_MEM_HOST_PINNED
    else:
        K, V, space = dev(Kh), dev(Vh), ig.IG_MEM_DEVICE
    d = desc_of(c)
    x, W, idx, q = dev(c.x), dev(c.W_in), dev(c.idx), dev(c.q)
    A_p = dev(c.A_p) if w.rope else None
    pos = dev(c.pos) if w.rope else None
    wq = torch.empty(ig.ig_wq_bytes(d), dtype=torch.uint8, device="cuda")
    slab = torch.empty(ig.ig_slab_bytes(d), dtype=torch.uint8, device="cuda")
    ctx.ig_wq_build(d, W, idx, wq)
    ctx.ig_slab_build(d, K, space, idx, slab)
    sel_idx = torch.zeros((BH, N), dtype=torch.int32, device="cuda")
    sel_cnt = torch.zeros((BH,), dtype=torch.int32, device="cuda")
    counters = torch.zeros((BH, N), dtype=torch.int32, device="cuda")
    victim = torch.zeros((BH,), dtype=torch.int32, device="cuda")
    ref_counters = np.zeros((BH, N), np.int32)
    if w.rope:
        q_p = o.project_rope(c.f32("x"), c.f32("W_in"), c.pos, c.A, c.idx)
    else:
        q_p = o.project(c.f32("x"), c.f32("W_in"), c.idx)
    for step in range(T):
        ctx.ig_speculate(d, x, wq, None, A_p, pos, slab, sel_idx, N, sel_cnt, None)
        ctx.ig_pool_touch(d, sel_idx, N, sel_cnt, counters, 3)          # tiny saturation value: halvings happen
        ctx.ig_pool_victim(d, counters, victim)
        kn = (rng.standard_normal((w.B, w.H, w.d)) * 2).astype(np.float16)
        vn = rng.standard_normal((w.B, w.H, w.d)).astype(np.float16)
        ctx.ig_pool_replace(d, victim, dev(kn), dev(vn), idx, slab, K, V, space, counters)
        torch.cuda.synchronize()
        assert ctx.ig_check_status() == 0
        # oracle on the mirror
        s = o.scan(q_p, np.ascontiguousarray(Kh, dtype=np.float32), c.idx, c.scale)
        r_idx, r_cnt = o.select(s, w.alpha)
        ref = OracleResult(q_p, s, r_idx, r_cnt, None, None, None, None)
        g_idx, g_cnt = sel_idx.cpu().numpy(), sel_cnt.cpu().numpy()
        slack = compare_selection(g_idx, g_cnt, ref, w.alpha)
        # the counters follow the lists that were prefetched; the oracle's own lists are used, which
        # are the GPU's whenever no score sits within 1e-3 of a threshold (true for these seeds)
        assert slack == 0, "a score inside the threshold band: pick another seed for this exact comparison"
        o.pool_touch(ref_counters, r_idx, r_cnt, N, counter_max=3)
        vic = o.pool_victim(ref_counters, N)
        assert np.array_equal(victim.cpu().numpy(), vic), step
        for i in range(BH):
            b, h = divmod(i, w.H)
            Kh[b, h, vic[i]] = kn[b, h]
            Vh[b, h, vic[i]] = vn[b, h]
            ref_counters[i, vic[i]] = 0
        assert np.array_equal(counters.cpu().numpy(), ref_counters), step
        assert np.array_equal(K.cpu().numpy(), Kh) and np.array_equal(V.cpu().numpy(), Vh), step
        print(f"  step {step}: victims {vic[:4]}..., in-band differences {slack}", flush=True)
    # the partial key cache followed the replacements: one more rehearsal against the mirror
    ctx.ig_speculate(d, x, wq, None, A_p, pos, slab, sel_idx, N, sel_cnt, None)
    torch.cuda.synchronize()
    s = o.scan(q_p, np.ascontiguousarray(Kh, dtype=np.float32), c.idx, c.scale)
    r_idx, r_cnt = o.select(s, w.alpha)
    compare_selection(sel_idx.cpu().numpy(), sel_cnt.cpu().numpy(),
                      OracleResult(q_p, s, r_idx, r_cnt, None, None, None, None), w.alpha)


def test_error_paths(ctx):
    import ctypes
    import paper_2406_19707_amd as ig
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    p = buf.data_ptr()
    d = ig.IgDesc(B=1, H=2, d=128, r=38, N=64)
    assert ctx.call("ig_pool_touch", ctypes.byref(d), p, 64, p, p, 0, 0) == ig.IG_EINVAL
    assert ctx.call("ig_pool_touch", ctypes.byref(d), p, 64, p, None, 255, 0) == ig.IG_EINVAL
    assert ctx.call("ig_pool_victim", ctypes.byref(d), None, p, 0) == ig.IG_EINVAL
    assert ctx.call("ig_pool_replace", ctypes.byref(d), None, p, p, p, p, p, p, 0, None, 0) == ig.IG_EINVAL
    # victims outside the pool are skipped, nothing is written
    vic = torch.tensor([-1, 64], dtype=torch.int32, device="cuda")
    pool = torch.zeros((2, 64, 128), dtype=torch.float16, device="cuda")
    new = torch.ones((1, 2, 128), dtype=torch.float16, device="cuda")
    slab = torch.zeros(ig.ig_slab_bytes(d), dtype=torch.uint8, device="cuda")
    idx = torch.zeros((2, 38), dtype=torch.int32, device="cuda")
    ctx.ig_pool_replace(d, vic, new, new, idx, slab, pool, pool, ig.IG_MEM_DEVICE, None)
    torch.cuda.synchronize()
    assert not pool.any() and not slab.any()


@pytest.mark.parametrize("policy_name", ["counter", "fifo", "lru"])
@pytest.mark.parametrize("cfg,shape,gain,N,T,host_pool", [
    (2, dict(B=2, H=4), 6.0, 1024, 6, False),
    (4, dict(B=2, H=2), 6.0, 600, 5, True),
])
def test_full_cache_decoding_under_each_policy(ctx, policy_name, cfg, shape, gain, N, T, host_pool):
    """The three victim selection policies of Section 4.4 / Table 2 through ig_pool_touch_policy,
    ig_pool_victim and ig_pool_replace_policy: per-slot state, victims and pools bit-exact against
    the oracle's counter / FIFO / LRU bookkeeping, step by step."""
    import paper_2406_19707_amd as ig
    from ig_gpu import desc_of, dev
    policy = {"counter": ig.IG_POLICY_COUNTER, "fifo": ig.IG_POLICY_FIFO, "lru": ig.IG_POLICY_LRU}[policy_name]
    w = wl.shrink(wl.WORKLOADS[cfg], N=N, heavy_count=8, pool="hbm", **shape)
    c = make_case(w, gain=gain)
    print(f"case {w.name} B{w.B} H{w.H} N{N} steps {T} host_pool {host_pool} policy {policy_name}", flush=True)
    BH = w.B * w.H
    rng = np.random.default_rng(123)
    Kh, Vh = c.Kt.copy(), c.V.copy()
    if host_pool:
        K, V, space = torch.from_numpy(Kh.copy()).pin_memory(), torch.from_numpy(Vh.copy()).pin_memory(), ig.IG_MEM_HOST_PINNED
    else:
        K, V, space = dev(Kh), dev(Vh), ig.IG_MEM_DEVICE
    d = desc_of(c)
    x, W, idx = dev(c.x), dev(c.W_in), dev(c.idx)
    wq = torch.empty(ig.ig_wq_bytes(d), dtype=torch.uint8, device="cuda")
    slab = torch.empty(ig.ig_slab_bytes(d), dtype=torch.uint8, device="cuda")
    ctx.ig_wq_build(d, W, idx, wq)
    ctx.ig_slab_build(d, K, space, idx, slab)
    sel_idx = torch.zeros((BH, N), dtype=torch.int32, device="cuda")
    sel_cnt = torch.zeros((BH,), dtype=torch.int32, device="cuda")
    victim = torch.zeros((BH,), dtype=torch.int32, device="cuda")
    # counter: zeros; FIFO / LRU: the prompt's entries carry their token positions
    ref_state = np.zeros((BH, N), np.int32) if policy_name == "counter" else np.tile(np.arange(N, dtype=np.int32), (BH, 1))
    state = torch.from_numpy(ref_state.copy()).cuda()
    q_p = o.project(c.f32("x"), c.f32("W_in"), c.idx)
    victims_seen = []
    for step in range(T):
        t_use, t_ins = 2 * (N + step), 2 * (N + step) + 1
        ctx.ig_speculate(d, x, wq, None, None, None, slab, sel_idx, N, sel_cnt, None)
        ctx.ig_pool_touch_policy(d, policy, sel_idx, N, sel_cnt, state, 3 if policy_name == "counter" else t_use)
        ctx.ig_pool_victim(d, state, victim)
        kn = (rng.standard_normal((w.B, w.H, w.d)) * 2).astype(np.float16)
        vn = rng.standard_normal((w.B, w.H, w.d)).astype(np.float16)
        ctx.ig_pool_replace_policy(d, policy, victim, dev(kn), dev(vn), idx, slab, K, V, space, state, t_ins)
        torch.cuda.synchronize()
        assert ctx.ig_check_status() == 0
        s = o.scan(q_p, np.ascontiguousarray(Kh, dtype=np.float32), c.idx, c.scale)
        r_idx, r_cnt = o.select(s, w.alpha)
        slack = compare_selection(sel_idx.cpu().numpy(), sel_cnt.cpu().numpy(),
                                  OracleResult(q_p, s, r_idx, r_cnt, None, None, None, None), w.alpha)
        assert slack == 0, "a score inside the threshold band: pick another seed for this exact comparison"
        if policy_name == "counter":
            o.pool_touch(ref_state, r_idx, r_cnt, N, counter_max=3)
            vic = o.pool_victim(ref_state, N)
        else:
            if policy_name == "lru":
                o.pool_touch_lru(ref_state, r_idx, r_cnt, N, now=t_use)
            vic = o.pool_victim_oldest(ref_state, N)
        assert np.array_equal(victim.cpu().numpy(), vic), step
        for i in range(BH):
            b, h = divmod(i, w.H)
            Kh[b, h, vic[i]] = kn[b, h]
            Vh[b, h, vic[i]] = vn[b, h]
            ref_state[i, vic[i]] = 0 if policy_name == "counter" else t_ins
        assert np.array_equal(state.cpu().numpy(), ref_state), step
        assert np.array_equal(K.cpu().numpy(), Kh) and np.array_equal(V.cpu().numpy(), Vh), step
        victims_seen.append(vic.copy())
    if policy_name == "fifo":        # FIFO walks through the prompt from its first token, used or not
        assert all(np.all(v == k) for k, v in enumerate(victims_seen))


def test_policy_error_paths(ctx):
    import ctypes
    import paper_2406_19707_amd as ig
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    p = buf.data_ptr()
    d = ig.IgDesc(B=1, H=2, d=128, r=38, N=64)
    assert ctx.call("ig_pool_touch_policy", ctypes.byref(d), 7, p, 64, p, p, 1, 0) == ig.IG_EINVAL
    assert ctx.call("ig_pool_touch_policy", ctypes.byref(d), ig.IG_POLICY_LRU, p, 64, p, None, 1, 0) == ig.IG_EINVAL
    assert ctx.call("ig_pool_touch_policy", ctypes.byref(d), ig.IG_POLICY_FIFO, p, 64, p, p, 1, 0) == ig.IG_OK
    assert ctx.call("ig_pool_replace_policy", ctypes.byref(d), 9, p, p, p, p, p, p, p, 0, p, 1, 0) == ig.IG_EINVAL
    assert ctx.call("ig_pool_replace_policy", ctypes.byref(d), ig.IG_POLICY_LRU, p, p, p, p, p, p, p, 0, None, 1, 0) == ig.IG_EINVAL
