"""HIP-graph replays of the per-layer call sequences (one stream, two streams with fork/join events,
and the joint launch of ig_layer_step) against the eager result: every sequence is captured once and
replayed several times with eager work and synchronisation between the replays, and every replay
must reproduce the eager attention output, index lists and fetched rows bit for bit."""
import pytest
import torch

import ig_workloads as wl

pytestmark = pytest.mark.gpu


def _capture(fn):
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        fn()                                   # warm-up outside capture (workspaces are sized here)
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=s):
        fn()
    return g


@pytest.mark.parametrize("cfg,kw", [(2, dict(B=4, H=8, N=2048)), (3, dict(B=2, H=8, N=1500))])
def test_graph_replays_match_eager(cfg, kw):
    import paper_2406_19707_amd as ig
    from paper_2406_19707_amd.pipeline import Rehearsal
    w = wl.shrink(wl.WORKLOADS[cfg], heavy_count=16, **kw)
    ctx = ig.Context(0)
    R = Rehearsal(ctx, w, gain=12.0, layers=5, host_layers=1, log=lambda *a: None)
    print(f"graph replay case {w.name} B{w.B} H{w.H} N{w.N} rope={w.rope}", flush=True)
    R._use(0)
    R.step_one_pass()
    torch.cuda.synchronize()
    assert ctx.ig_check_status() == ig.IG_OK
    last = (R.L - 1) % R.n_sets
    ref_out = R.out.clone()
    ref_idx, ref_cnt = R.sets[last]["sel_idx"].clone(), R.sets[last]["sel_cnt"].clone()
    n_max = int(ref_cnt.max().item())
    ref_K = R.sets[last]["K_sel"][:, :n_max].clone()
    assert n_max >= 1
    for name, fn in (("one stream", R.step_one_pass), ("two streams", R.step_two_stream), ("joint launch", R.step_joint)):
        g = _capture(fn)
        for rep in range(3):
            # eager work and a synchronisation between the replays; the outputs are wiped first
            R._use(0)
            R.speculate(0)
            R.out.zero_()
            for st in R.sets:
                st["sel_cnt"].zero_()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            st = R.sets[last]
            assert torch.equal(R.out, ref_out), (name, rep)
            assert torch.equal(st["sel_cnt"], ref_cnt), (name, rep)
            cnt = ref_cnt.cpu()
            idx_ok = all(torch.equal(st["sel_idx"][i, :cnt[i]], ref_idx[i, :cnt[i]]) for i in range(0, ref_cnt.numel(), 7))
            assert idx_ok, (name, rep)
            rows_ok = all(torch.equal(st["K_sel"][i, :cnt[i]], ref_K[i, :cnt[i]]) for i in range(0, ref_cnt.numel(), 7))
            assert rows_ok, (name, rep)
        print(f"  {name}: 3 replays equal the eager result", flush=True)
    assert ctx.ig_check_status() == ig.IG_OK
    R.side_ctx.close()
    ctx.close()


def test_workspace_growth_under_capture_is_refused():
    """A call that would have to allocate a workspace while its stream is being captured returns an
    error (and leaves the capture valid) instead of allocating; after ig_reserve the same call is
    captured and replays correctly."""
    import paper_2406_19707_amd as ig
    from ig_case import make_case
    from ig_gpu import Uploaded
    w = wl.shrink(wl.WORKLOADS[2], B=2, H=8, N=1024, heavy_count=8)
    c = make_case(w, gain=12.0)
    build_ctx = ig.Context(0)
    up = Uploaded(build_ctx, c)                      # slab and weight blob built with another context
    ctx = ig.Context(0)                              # fresh: no workspace yet
    d = up.desc
    BH = w.B * w.H
    sel_idx = torch.zeros((BH, c.N), dtype=torch.int32, device="cuda")
    sel_cnt = torch.zeros(BH, dtype=torch.int32, device="cuda")
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=s):
        with pytest.raises(ig.IgError) as e:
            ctx.ig_speculate(d, up.x, up.wq, up.bias, up.A_p, up.pos, up.slab, sel_idx, c.N, sel_cnt, None)
        assert e.value.code == ig.IG_EINVAL and "ig_reserve" in str(e.value)
        sel_cnt.fill_(7)                             # the capture is still usable
    g.replay()
    torch.cuda.synchronize()
    assert int(sel_cnt[0]) == 7
    ctx.ig_reserve(d)
    ref_idx, ref_cnt = torch.zeros_like(sel_idx), torch.zeros_like(sel_cnt)
    build_ctx.ig_speculate(d, up.x, up.wq, up.bias, up.A_p, up.pos, up.slab, ref_idx, c.N, ref_cnt, None)
    torch.cuda.synchronize()
    g2 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g2, stream=s):
        ctx.ig_speculate(d, up.x, up.wq, up.bias, up.A_p, up.pos, up.slab, sel_idx, c.N, sel_cnt, None)
    for _ in range(2):
        sel_cnt.zero_()
        torch.cuda.synchronize()
        g2.replay()
        torch.cuda.synchronize()
        assert torch.equal(sel_cnt, ref_cnt)
    ctx.close()
    build_ctx.close()
