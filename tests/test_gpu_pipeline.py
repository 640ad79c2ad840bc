"""GPU parity of the decode-step drivers (paper_2406_19707_amd/pipeline.py) against their serial
form and the CPU oracle, layer by layer:

* Rehearsal.step_overlapped -- the host-pool pipeline of Section 4.1 / Fig. 3(d): the selected rows
  of layer l cross PCIe on a side stream while the main stream rehearses layer l+1 and attends
  layer l-1, over two buffer sets and cross-stream events;
* Rehearsal.decode -- the growing-cache loop (Section 2.1, Section 4.3): per layer rehearsal,
  prefetch, attention over the cached tokens plus the token being decoded, then the append; first
  layer dense or not.
"""
import numpy as np
import pytest
import torch

import ig_workloads as wl
from ig_case import OracleResult, compare_selection
from oracle import ig_oracle as o

pytestmark = pytest.mark.gpu


def f32(t):
    return np.ascontiguousarray(t.float().cpu().numpy(), dtype=np.float32)


def oracle_layer(R, l, N, alpha, k_new=None, v_new=None):
    """The oracle on layer l of a Rehearsal, over its first N cached tokens."""
    w = R.w
    p = l % R.n_pool
    x, Kt, V, q = f32(R.x[l]), f32(R.K[p]), f32(R.V[p]), f32(R.q[l])
    Wf = np.ascontiguousarray(R.W_host, dtype=np.float32)
    if w.rope:
        q_p = o.project_rope(x, Wf, np.full(w.B, w.N, np.int32), R.A, R.idx_host)
    else:
        q_p = o.project(x, Wf, R.idx_host)
    s = o.scan(q_p, Kt, R.idx_host, R.desc.scale, N=N)
    sel_idx, sel_cnt = o.select(s, alpha)
    K_sel, V_sel = o.gather(Kt, sel_idx, sel_cnt), o.gather(V, sel_idx, sel_cnt)
    out = o.attend(q, K_sel, V_sel, sel_cnt, R.desc.scale,
                   None if k_new is None else f32(k_new), None if v_new is None else f32(v_new))
    return OracleResult(q_p, s, sel_idx, sel_cnt, K_sel, V_sel, out, None)


def snapshot(R):
    return dict(sel_idx=R.sel_idx.clone(), sel_cnt=R.sel_cnt.clone(), K_sel=R.K_sel.clone(),
                V_sel=R.V_sel.clone(), out=R.out.clone())


def check_against_oracle(R, snap, ref, alpha):
    w = R.w
    BH = w.B * w.H
    g_idx, g_cnt = snap["sel_idx"].cpu().numpy(), snap["sel_cnt"].cpu().numpy()
    slack = compare_selection(g_idx, g_cnt, ref, alpha)
    if slack == 0:
        Ks, Vs = f32(snap["K_sel"]), f32(snap["V_sel"])
        for i in range(BH):                      # rows beyond a list's count are not written
            n = int(ref.sel_cnt[i])
            assert np.array_equal(Ks[i, :n], ref.K_sel[i, :n]) and np.array_equal(Vs[i, :n], ref.V_sel[i, :n])
        err = np.abs(f32(snap["out"]).reshape(BH, w.d) - ref.out)
        assert np.all(err <= 2e-2 + 1e-2 * np.abs(ref.out)), err.max()
    return slack


@pytest.mark.parametrize("cfg,B,H,N,L,sets,gain", [
    (4, 2, 8, 2048, 6, 2, 12.0),     # OPT-30B-like, folded skew, pinned host pool, two buffer sets
    (5, 1, 8, 6000, 5, 2, 30.0),     # long-context-like, rotary, pairs split over workgroups
    (4, 2, 8, 1000, 7, 3, 12.0),     # three buffer sets
])
def test_overlapped_host_pool_step_matches_serial_and_oracle(cfg, B, H, N, L, sets, gain):
    import paper_2406_19707_amd as ig
    from paper_2406_19707_amd.pipeline import Rehearsal
    w = wl.shrink(wl.WORKLOADS[cfg], B=B, H=H, N=N, n_cal=256, heavy_count=16)
    ctx = ig.Context(0)
    R = Rehearsal(ctx, w, gain=gain, layers=L, host_layers=L, sets=sets)
    assert R.host_pool and R.n_pool == L and all(k.is_pinned() for k in R.K)
    # serial reference: one layer at a time on one stream
    serial = []
    for l in range(L):
        R._use(l)
        R.layer(l)
        torch.cuda.synchronize()
        serial.append(snapshot(R))
    # the pipelined step, twice in a row (the second starts on the first one's leftovers)
    for rep in range(2):
        for st in R.sets:
            for t in st.values():
                t.fill_(-1 if t.dtype == torch.int32 else 7)
        piped = {}
        R.step_overlapped(after_layer=lambda l: piped.__setitem__(l, snapshot(R)))
        torch.cuda.synchronize()
        assert ctx.ig_check_status() == ig.IG_OK and R.side_ctx.ig_check_status() == ig.IG_OK
        assert sorted(piped) == list(range(L))
        for l in range(L):
            n = serial[l]["sel_cnt"]
            assert torch.equal(piped[l]["sel_cnt"], n), (rep, l)
            assert torch.equal(piped[l]["out"], serial[l]["out"]), (rep, l)
            for i in range(w.B * w.H):
                k = int(n[i])
                assert torch.equal(piped[l]["sel_idx"][i, :k], serial[l]["sel_idx"][i, :k])
                assert torch.equal(piped[l]["K_sel"][i, :k], serial[l]["K_sel"][i, :k])
                assert torch.equal(piped[l]["V_sel"][i, :k], serial[l]["V_sel"][i, :k])
    # every layer of the pipelined step against the oracle
    fracs = []
    for l in range(L):
        ref = oracle_layer(R, l, w.N, w.alpha)
        check_against_oracle(R, piped[l], ref, w.alpha)
        fracs.append(ref.sel_cnt.mean() / w.N)
    print(f"selected fraction per layer: {np.round(fracs, 4)}", flush=True)
    assert 0 < min(fracs) and max(fracs) < 1          # a real selection, not the degenerate cases
    ctx.close()


@pytest.mark.parametrize("cfg,B,H,N,host,dense_first,gain", [
    (2, 2, 4, 1020, False, True, 8.0),     # HBM pool, first layer dense, crosses a tile boundary
    (2, 2, 4, 1020, False, False, 8.0),
    (3, 2, 4, 700, False, True, 20.0),     # rotary
    (4, 2, 4, 600, True, True, 8.0),       # pinned host pool
])
def test_decode_loop_matches_oracle_at_every_length(cfg, B, H, N, host, dense_first, gain):
    import paper_2406_19707_amd as ig
    from paper_2406_19707_amd.pipeline import Rehearsal
    T, L = 5, 3
    w = wl.shrink(wl.WORKLOADS[cfg], B=B, H=H, N=N, n_cal=256, heavy_count=8,
                  pool="host" if host else "hbm")
    ctx = ig.Context(0)
    R = Rehearsal(ctx, w, gain=gain, layers=L, host_layers=L, extra_tokens=T)
    snaps = {}
    R.decode(T, dense_first_layer=dense_first, after_layer=lambda s, l: snaps.__setitem__((s, l), snapshot(R)))
    torch.cuda.synchronize()
    assert ctx.ig_check_status() == ig.IG_OK
    assert len(snaps) == T * L
    # after the loop every pool holds the original cache followed by T copies of the new token
    k_new, v_new = R.k_new, R.v_new
    for l in range(L):
        K, V = R.K[l], R.V[l]
        for t in range(T):
            assert torch.equal(K[:, :, N + t].to("cuda"), k_new) and torch.equal(V[:, :, N + t].to("cuda"), v_new)
    # the oracle on the cache as it was at (step, layer): N + step tokens, plus the token being decoded
    for (s, l), snap in snaps.items():
        alpha = float("inf") if (dense_first and l == 0) else w.alpha
        ref = oracle_layer(R, l, N + s, alpha, k_new, v_new)
        if alpha == float("inf"):
            assert np.all(ref.sel_cnt == N + s)
        check_against_oracle(R, snap, ref, alpha)
    ctx.close()


@pytest.mark.parametrize("cfg,B,H,N,L,gain", [
    (2, 2, 8, 2500, 3, 12.0),      # HBM pool, folded skew
    (5, 1, 8, 6000, 3, 30.0),      # rotary query, pinned host pool
])
def test_host_speculation_step_matches_device_step_and_oracle(cfg, B, H, N, L, gain):
    """Section 6.2: partial key cache in host memory, speculation on the CPU.  Same lists, rows and
    attention output as the all-GPU layer, bit for bit, and both against the oracle."""
    import paper_2406_19707_amd as ig
    from paper_2406_19707_amd.pipeline import Rehearsal
    w = wl.shrink(wl.WORKLOADS[cfg], B=B, H=H, N=N, n_cal=256, heavy_count=16)
    ctx = ig.Context(0)
    R = Rehearsal(ctx, w, gain=gain, layers=L, host_layers=L)
    serial = []
    for l in range(L):
        R._use(0)
        R.layer(l)
        torch.cuda.synchronize()
        serial.append(snapshot(R))
    R.host_speculation_setup(slab_layers=L)
    for st in R.sets:
        for t in st.values():
            t.fill_(-1 if t.dtype == torch.int32 else 7)
    R._use(0)
    hosted = {}
    R.step_host_speculation(threads=4, after_layer=lambda l: hosted.__setitem__(l, snapshot(R)))
    torch.cuda.synchronize()
    assert ctx.ig_check_status() == ig.IG_OK
    for l in range(L):
        n = serial[l]["sel_cnt"]
        assert torch.equal(hosted[l]["sel_cnt"], n), l
        assert torch.equal(hosted[l]["out"], serial[l]["out"]), l
        for i in range(w.B * w.H):
            k = int(n[i])
            assert torch.equal(hosted[l]["sel_idx"][i, :k], serial[l]["sel_idx"][i, :k])
            assert torch.equal(hosted[l]["K_sel"][i, :k], serial[l]["K_sel"][i, :k])
        ref = oracle_layer(R, l, w.N, w.alpha)
        check_against_oracle(R, hosted[l], ref, w.alpha)
    ctx.close()


@pytest.mark.parametrize("cfg,B,H,N,L,sets,gain", [
    (4, 2, 8, 2048, 6, 2, 12.0),
    (5, 1, 8, 6000, 5, 3, 30.0),
])
def test_native_overlapped_step_matches_the_serial_layers(cfg, B, H, N, L, sets, gain):
    """ig_decode_step_overlapped (the two-stream pipeline issued by the library) against one layer at
    a time on one stream: every layer's output bit for bit, twice in a row, and the lists and rows
    the last `sets` layers left in the buffer sets."""
    import paper_2406_19707_amd as ig
    from paper_2406_19707_amd.pipeline import Rehearsal
    w = wl.shrink(wl.WORKLOADS[cfg], B=B, H=H, N=N, n_cal=256, heavy_count=16)
    ctx = ig.Context(0)
    R = Rehearsal(ctx, w, gain=gain, layers=L, host_layers=L, sets=sets)
    serial = []
    for l in range(L):
        R._use(l)
        R.layer(l)
        torch.cuda.synchronize()
        serial.append(snapshot(R))
    for rep in range(2):
        for st in R.sets:
            for t in st.values():
                t.fill_(-1 if t.dtype == torch.int32 else 7)
        R.step_overlapped_native()
        torch.cuda.synchronize()
        assert ctx.ig_check_status() == ig.IG_OK
        for l in range(L):
            assert torch.equal(R.outs[l], serial[l]["out"]), (rep, l)
        for l in range(L - sets, L):
            st = R.sets[l % sets]
            n = serial[l]["sel_cnt"]
            assert torch.equal(st["sel_cnt"], n), (rep, l)
            for i in range(w.B * w.H):
                k = int(n[i])
                assert torch.equal(st["sel_idx"][i, :k], serial[l]["sel_idx"][i, :k])
                assert torch.equal(st["K_sel"][i, :k], serial[l]["K_sel"][i, :k])
                assert torch.equal(st["V_sel"][i, :k], serial[l]["V_sel"][i, :k])
    # the library refuses what it cannot order
    with pytest.raises(ig.IgError):
        ctx.ig_decode_step_overlapped(R.desc, R._native_layers, R.wq, None, R.A_p, R.pos, R.space,
                                      R._native_sets, R.stride, R.side, R.side)
    ctx.close()


def test_native_overlapped_step_error_paths():
    import ctypes
    import paper_2406_19707_amd as ig
    ctx = ig.Context(0)
    d = ig.IgDesc(B=1, H=2, d=128, r=38, N=64)
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    p = buf.data_ptr()
    layers = (ig.IgLayerIO * 1)(ig.IgLayerIO(x=p, slab=p, q=p, Kpool=p, Vpool=p, k_new=None, v_new=None, out=p))
    sets = (ig.IgBufferSet * 2)(ig.IgBufferSet(sel_idx=p, sel_cnt=p, K_sel=p, V_sel=p),
                                ig.IgBufferSet(sel_idx=p, sel_cnt=p, K_sel=p, V_sel=None))
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    def call(n_layers=1, n_sets=2, main=s1.cuda_stream, side=s2.cuda_stream, la=ctypes.addressof(layers)):
        return ctx.call("ig_decode_step_overlapped", ctypes.byref(d), n_layers, la, p, 0, 0, 0, ig.IG_MEM_DEVICE,
                        n_sets, ctypes.addressof(sets), 64, main, side)
    assert call(n_layers=0) == ig.IG_EINVAL
    assert call(n_sets=1) == ig.IG_EINVAL
    assert call(la=0) == ig.IG_EINVAL
    assert call(side=s1.cuda_stream) == ig.IG_EINVAL and "differ" in ctx.last_error()
    assert call() == ig.IG_EINVAL and "NULL member" in ctx.last_error()     # second set lacks V_sel
    torch.cuda.synchronize()
    ctx.close()
