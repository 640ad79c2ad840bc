"""The allocation-free attention entry point against the ordinary one (GPU).

ig_sparse_attention_static keeps its slice states and arrival counters in the library's static
device array.  Two calls in a row on one context that never reserved or grew a workspace, the
second with a smaller input, each compared with ig_sparse_attention (same kernel: bit for bit)
and with the CPU oracle's attention to the usual bar."""
import ctypes

import numpy as np
import pytest
import torch

import ig_workloads as wl
from ig_case import make_case, run_oracle
from ig_gpu import Uploaded, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ig():
    import paper_2406_19707_amd as ig
    return ig


def _lists_and_rows(ig, ctx, c, ref):
    """Oracle lists uploaded, rows fetched by the ordinary gather (on the ordinary context)."""
    w = c.w
    up = Uploaded(ctx, c)
    BH = w.B * w.H
    stride = c.N
    tdt = torch.float32 if w.dtype == "f32" else torch.float16
    sel_idx, sel_cnt = dev(ref.sel_idx.astype(np.int32)), dev(ref.sel_cnt.astype(np.int32))
    K_sel = torch.zeros((BH, stride, w.d), dtype=tdt, device="cuda")
    V_sel = torch.zeros_like(K_sel)
    ctx.ig_gather_kv(up.desc, up.K, up.V, up.space, sel_idx, stride, sel_cnt, K_sel, V_sel)
    torch.cuda.synchronize()
    return up, sel_cnt, K_sel, V_sel, stride, tdt


def test_static_scratch_attention_matches_the_ordinary_entry_point(ig):
    ctx = ig.Context(0)          # gathers, and the ordinary attention
    bare = ig.Context(0)         # only ever sees the allocation-free call
    assert bare.ig_workspace_bytes() == 0
    # first call: every token selected (16 slices per list, so the slice states and counters are
    # used); second call: fewer heads, shorter and ragged lists, plus the token being decoded
    first = make_case(wl.shrink(wl.WORKLOADS[2], B=2, H=8, N=2048), gain=1.0)
    second = make_case(wl.shrink(wl.WORKLOADS[2], B=1, H=4, N=700), gain=24.0)
    for c, with_new in ((first, False), (second, True)):
        w = c.w
        ref = run_oracle(c)
        up, sel_cnt, K_sel, V_sel, stride, tdt = _lists_and_rows(ig, ctx, c, ref)
        k_new, v_new = (up.k_new, up.v_new) if with_new else (None, None)
        out_a = torch.full((w.B, w.H, w.d), float("nan"), dtype=tdt, device="cuda")
        out_b = torch.full_like(out_a, float("nan"))
        ctx.ig_sparse_attention(up.desc, up.q, K_sel, V_sel, sel_cnt, stride, k_new, v_new, out_a)
        bare.ig_sparse_attention_static(up.desc, up.q, K_sel, V_sel, sel_cnt, stride, k_new, v_new, out_b)
        torch.cuda.synchronize()
        assert bare.ig_check_status() == ig.IG_OK
        assert bare.ig_workspace_bytes() == 0, "the allocation-free call grew a workspace"
        assert torch.equal(out_a, out_b)
        want = ref.out_new if with_new else ref.out
        got = out_b.float().cpu().numpy().reshape(-1, w.d)
        assert np.all(np.abs(got - want) <= 2e-2 + 1e-2 * np.abs(want)), np.abs(got - want).max()
    assert first.w.B * first.w.H > second.w.B * second.w.H
    assert int(run_oracle(first).sel_cnt.max()) == 2048      # multi-slice lists were in play
    # sizes beyond the static array are refused before anything is launched
    big = ig.IgDesc(B=64, H=64, d=128, r=38, N=16)
    one = torch.zeros(16, dtype=torch.float16, device="cuda")
    cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    rc = bare.call("ig_sparse_attention_static", ctypes.byref(big), one.data_ptr(), one.data_ptr(), one.data_ptr(),
                   cnt.data_ptr(), 16, None, None, one.data_ptr(), None)
    assert rc == ig.IG_ECAPACITY and "static scratch" in bare.last_error()
    bare.close()
    ctx.close()
