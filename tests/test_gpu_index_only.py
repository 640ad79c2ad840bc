"""GPU parity of the index-only partial weight (Section 6.2 "Memory Consumption": only the column
indices are stored, the columns come from the full skewed query weight at run time):
ig_project_indexed / ig_speculate_indexed against the CPU oracle, which projects from the full
weight and the index table by definition.  Same bars as the stored-blob path: partial queries and
scores to float32 summation order, index lists bit-exact outside the 1e-3 band at the threshold."""
import numpy as np
import pytest
import torch

import ig_workloads as wl
from ig_case import make_case, run_oracle, compare_selection

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_2406_19707_amd as ig
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = ig.Context(0)
    yield c
    c.close()


def check_indexed(ctx, c, alpha=None):
    import paper_2406_19707_amd as ig
    from ig_gpu import desc_of, dev
    w = c.w
    alpha = w.alpha if alpha is None else alpha
    print(f"index-only case {w.name} B{w.B} H{w.H} d{w.d} N{c.N}/{c.N_cap} r{c.r} {w.dtype} "
          f"bias={c.bias_in is not None}", flush=True)
    ref = run_oracle(c, alpha, attend=False)
    d = desc_of(c, alpha)
    x, W, idx, bias, K = dev(c.x), dev(c.W_in), dev(c.idx), dev(c.bias_in), dev(c.Kt)
    slab = torch.empty(ig.ig_slab_bytes(d), dtype=torch.uint8, device="cuda")
    ctx.ig_slab_build(d, K, ig.IG_MEM_DEVICE, idx, slab)
    BH = w.B * w.H
    q_p = torch.full((w.B, w.H, c.r), float("nan"), device="cuda")
    scores = torch.full((w.B, w.H, c.N), float("nan"), device="cuda")
    sel_idx = torch.full((BH, c.N), -1, dtype=torch.int32, device="cuda")
    sel_cnt = torch.full((BH,), -1, dtype=torch.int32, device="cuda")
    ctx.ig_project_indexed(d, x, W, idx, bias, q_p)
    ctx.ig_speculate_indexed(d, x, W, idx, bias, slab, sel_idx, c.N, sel_cnt, scores)
    # twice: the sums are taken in a fixed order
    q_p2, sel_idx2, sel_cnt2 = torch.zeros_like(q_p), torch.full_like(sel_idx, -1), torch.zeros_like(sel_cnt)
    ctx.ig_project_indexed(d, x, W, idx, bias, q_p2)
    ctx.ig_speculate_indexed(d, x, W, idx, bias, slab, sel_idx2, c.N, sel_cnt2, None)
    torch.cuda.synchronize()
    assert ctx.ig_check_status() == ig.IG_OK
    assert torch.equal(q_p, q_p2) and torch.equal(sel_idx, sel_idx2) and torch.equal(sel_cnt, sel_cnt2)
    qtol = 2e-5 * max(1.0, np.abs(ref.q_p).max())
    assert np.abs(q_p.cpu().numpy() - ref.q_p).max() <= qtol
    stol = 1e-4 * max(1.0, np.abs(ref.s).max())
    assert np.abs(scores.cpu().numpy() - ref.s).max() <= stol
    slack = compare_selection(sel_idx.cpu().numpy(), sel_cnt.cpu().numpy(), ref, alpha)
    print(f"  selected fraction {ref.sel_cnt.mean() / c.N:.4f}, in-band differences {slack}", flush=True)


def test_cfg1_f32(ctx):
    check_indexed(ctx, make_case(wl.WORKLOADS[1], gain=8.0))


@pytest.mark.parametrize("B,H,N,bias", [(3, 4, 1999, False), (8, 6, 700, True), (1, 2, 64, False)])
def test_cfg2_shape_f16(ctx, B, H, N, bias):
    w = wl.shrink(wl.WORKLOADS[2], B=B, H=H, N=N, heavy_count=min(20, N))
    check_indexed(ctx, make_case(w, gain=6.0, bias=bias))


@pytest.mark.parametrize("B", [9, 20, 40])
def test_more_sequences_than_one_batch_block(ctx, B):
    w = wl.shrink(wl.WORKLOADS[4], B=B, H=2, N=600, pool="hbm")
    check_indexed(ctx, make_case(w, gain=6.0))


def test_head_dimension_256_f16_and_64_f32(ctx):
    w = wl.shrink(wl.WORKLOADS[2], B=2, H=3, d=256, N=700, n_cal=384, heavy_count=8)
    check_indexed(ctx, make_case(w, gain=4.0))
    w = wl.shrink(wl.WORKLOADS[1], B=5, H=8, N=900, heavy_count=10)                 # d = 64 floats: 256-byte rows
    check_indexed(ctx, make_case(w, gain=8.0, bias=True))


def test_small_and_non_power_of_two_head_dimensions(ctx):
    # d = 8 halves: one 16-byte piece per row (64 rows per wave-wide load); d = 24 and 40 halves:
    # 3 and 5 pieces, padded to 4 and 8 lanes
    for d_, H in ((8, 3), (24, 4), (40, 2)):
        w = wl.shrink(wl.WORKLOADS[2], B=2, H=H, d=d_, N=900, ratio=0.5, n_cal=96, heavy_count=5)
        check_indexed(ctx, make_case(w, gain=2.0))


def test_matrix_core_path_column_blocks_across_heads_and_many_sequences(ctx):
    # half precision with D % 128 == 0 runs on the matrix cores in 128-column blocks: d = 64 puts
    # two heads into a block, d = 32 four; 70 sequences need two passes of four 16-row batch blocks
    w = wl.shrink(wl.WORKLOADS[2], B=3, H=6, d=64, N=800, n_cal=128, heavy_count=8)
    check_indexed(ctx, make_case(w, gain=5.0, bias=True))
    w = wl.shrink(wl.WORKLOADS[2], B=70, H=8, d=32, N=300, n_cal=96, heavy_count=6)
    check_indexed(ctx, make_case(w, gain=4.0))


def test_all_columns(ctx):
    w = wl.shrink(wl.WORKLOADS[2], B=2, H=4, N=1100)
    check_indexed(ctx, make_case(w, gain=3.0, all_columns=True))


def test_wide_model_dimension_several_chunks(ctx):
    # D = 64 * 128 = 8192 with 2 sequences: K slices of 1024 rows, two staged chunks each
    w = wl.shrink(wl.WORKLOADS[2], B=2, H=64, N=520, n_cal=160, heavy_count=6)
    check_indexed(ctx, make_case(w, gain=96.0))


def test_error_paths(ctx):
    import paper_2406_19707_amd as ig
    from ig_gpu import desc_of, dev
    w = wl.shrink(wl.WORKLOADS[3], B=2, H=2, N=256)            # rotary model
    c = make_case(w, gain=8.0)
    d = desc_of(c)
    x, W, idx = dev(c.x), dev(c.W_in), dev(c.idx)
    q_p = torch.zeros((w.B, w.H, c.r), device="cuda")
    with pytest.raises(ig.IgError):
        ctx.ig_project_indexed(d, x, W, idx, None, q_p)          # rope == 1 is refused
    w = wl.shrink(wl.WORKLOADS[2], B=2, H=2, N=256)
    c = make_case(w, gain=6.0)
    d = desc_of(c)
    x, W, idx = dev(c.x), dev(c.W_in), dev(c.idx)
    with pytest.raises(ig.IgError):
        ctx.ig_project_indexed(d, x, W, None, None, q_p)         # missing index table
    with pytest.raises(ig.IgError):
        ctx.ig_project_indexed(d, x, W, idx, None, None)         # missing output
    torch.cuda.synchronize()
    assert ctx.ig_check_status() == ig.IG_OK
