"""GPU parity: the HIP path against the CPU oracle, element by element, through the C ABI.

Bars: index lists bit-exact except tokens whose float32 oracle score lies within 1e-3 of the oracle
threshold; gathered rows bit-exact; attention output within 2e-2 abs + 1e-2 rel for half-precision
KV (1e-4 / 1e-4 for float32); partial queries and scores to float32 summation-order error.
"""
import numpy as np
import pytest
import torch

import ig_workloads as wl
from ig_case import make_case, run_oracle, compare_selection
from oracle import ig_oracle as o

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_2406_19707_amd as ig
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = ig.Context(0)
    yield c
    c.close()


def check_case(ctx, c, alpha=None, host_pool=False, expect_fraction=None):
    from ig_gpu import run_gpu, run_gpu_on_lists
    w = c.w
    alpha = w.alpha if alpha is None else alpha
    print(f"case {w.name} B{w.B} H{w.H} d{w.d} N{c.N}/{c.N_cap} r{c.r} {w.dtype} rope={w.rope} "
          f"alpha={alpha} host_pool={host_pool}", flush=True)
    ref = run_oracle(c, alpha)
    got = run_gpu(ctx, c, alpha, host_pool=host_pool)
    assert got["status"] == 0
    BH = w.B * w.H
    # partial queries and scores: float32 accumulation order only
    qtol = 2e-5 * max(1.0, np.abs(ref.q_p).max()) * (8 if w.rope else 1)
    assert np.abs(got["q_p"] - ref.q_p).max() <= qtol
    stol = 1e-4 * max(1.0, np.abs(ref.s).max())
    assert np.abs(got["scores"] - ref.s).max() <= stol
    # index lists
    slack = compare_selection(got["sel_idx"], got["sel_cnt"], ref, alpha)
    frac = ref.sel_cnt.mean() / c.N
    print(f"  selected fraction {frac:.4f} (min {ref.sel_cnt.min()}, max {ref.sel_cnt.max()}), "
          f"in-band differences {slack}", flush=True)
    if expect_fraction:
        assert expect_fraction[0] <= frac <= expect_fraction[1]
    # gathered rows: bit-exact copies of the rows the GPU's own lists name
    Kt = c.Kt.reshape(BH, c.N_cap, w.d)
    V = c.V.reshape(BH, c.N_cap, w.d)
    for i in range(BH):
        n = got["sel_cnt"][i]
        rows = got["sel_idx"][i, :n]
        assert np.array_equal(got["K_sel"][i, :n], Kt[i, rows])
        assert np.array_equal(got["V_sel"][i, :n], V[i, rows])
        assert not got["K_sel"][i, n:].any() and not got["V_sel"][i, n:].any()   # untouched
    if got["K_one"] is not None:      # the one-pass prefetch + attention writes the same rows
        assert np.array_equal(got["K_one"], got["K_sel"]) and np.array_equal(got["V_one"], got["V_sel"])
    # attention on the GPU's own lists: comparable with the oracle's output when the lists agree
    atol, rtol = (1e-4, 1e-4) if w.dtype == "f32" else (2e-2, 1e-2)
    if slack == 0:
        for name, r_ in (("out", ref.out), ("out_new", ref.out_new), ("out_idx", ref.out),
                         ("out_one", ref.out), ("out_one_new", ref.out_new)):
            if got[name] is None:
                continue
            err = np.abs(got[name] - r_)
            assert np.all(err <= atol + rtol * np.abs(r_)), (name, err.max())
    # prefetch and attention fed with the oracle's lists (inputs flow oracle -> HIP path)
    fed = run_gpu_on_lists(ctx, c, got["up"], ref.sel_idx, ref.sel_cnt, host_pool)
    n_max = int(ref.sel_cnt.max())
    assert np.array_equal(fed["K_sel"][:, :n_max], ref.K_sel[:, :n_max])
    assert np.array_equal(fed["V_sel"][:, :n_max], ref.V_sel[:, :n_max])
    for name, r_ in (("out", ref.out), ("out_new", ref.out_new), ("out_idx", ref.out), ("out_one", ref.out)):
        if fed[name] is None:
            continue
        err = np.abs(fed[name] - r_)
        assert np.all(err <= atol + rtol * np.abs(r_)), ("oracle lists", name, err.max())
    return ref, got


def test_cfg1_single_layer_f32(ctx):
    # configs[0]: B1 H4 d64 N512 float32, r = 19, alpha 4; logit gain 8 puts the layer in the sparse regime
    check_case(ctx, make_case(wl.WORKLOADS[1], gain=8.0), expect_fraction=(0.01, 0.5))


def test_cfg1_literal_scale_selects_everything(ctx):
    ref, got = check_case(ctx, make_case(wl.WORKLOADS[1], gain=1.0))
    assert np.all(got["sel_cnt"] == 512)


def test_all_columns_and_infinite_alpha_is_dense_attention(ctx):
    w = wl.shrink(wl.WORKLOADS[1], B=2, N=300)
    c = make_case(w, all_columns=True)
    ref, got = check_case(ctx, c, alpha=float("inf"))
    assert np.all(got["sel_cnt"] == 300)
    q = torch.from_numpy(c.f32("q")).double().reshape(-1, 1, w.d)
    K = torch.from_numpy(c.f32("Kt")).double().reshape(-1, c.N_cap, w.d)[:, :300]
    V = torch.from_numpy(c.f32("V")).double().reshape(-1, c.N_cap, w.d)[:, :300]
    dense = torch.nn.functional.scaled_dot_product_attention(q, K, V, scale=c.scale)[:, 0].numpy()
    assert np.abs(got["out"] - dense).max() <= 1e-4


@pytest.mark.parametrize("N,N_cap", [(2048, 2048), (1999, 2048), (700, 1024), (1, 8), (700, 6000)])
def test_cfg2_shape_f16_fused_four_waves(ctx, N, N_cap):
    w = wl.shrink(wl.WORKLOADS[2], B=3, H=4, N=N, heavy_count=min(20, N))
    check_case(ctx, make_case(w, gain=6.0, N_cap=N_cap))


def test_cfg2_shape_with_bias_and_key_term_in_index(ctx):
    w = wl.shrink(wl.WORKLOADS[2], B=2, H=4, N=1500)
    check_case(ctx, make_case(w, gain=6.0, bias=True, use_keys_for_index=True))


@pytest.mark.parametrize("N", [3000, 6000])
def test_many_heads_fused_eight_and_sixteen_waves(ctx, N):
    # B*H = 128 pairs: N = 3000 -> 6 tiles (8-wave workgroups), N = 6000 -> 12 tiles (16-wave)
    w = wl.shrink(wl.WORKLOADS[2], B=8, H=16, d=32, N=N, heavy_count=30)
    check_case(ctx, make_case(w, gain=6.0))


@pytest.mark.parametrize("ratio,all_columns", [(0.6, False), (1.0, True)])
def test_wide_partial_queries_more_than_64_columns(ctx, ratio, all_columns):
    # r = 76 and r = 128: the partial query spans two per-lane registers and several channel blocks
    w = wl.shrink(wl.WORKLOADS[2], B=2, H=4, N=1100, ratio=ratio)
    check_case(ctx, make_case(w, gain=3.0, all_columns=all_columns))


def test_wide_partial_queries_long_sequence_tiled_path(ctx):
    w = wl.shrink(wl.WORKLOADS[5], B=1, H=2, N=9000, ratio=0.7)     # r = 89, one wave per tile
    check_case(ctx, make_case(w, gain=3.0))


def test_head_dimension_256_and_odd_head_count(ctx):
    w = wl.shrink(wl.WORKLOADS[2], B=2, H=3, d=256, N=700, n_cal=384, heavy_count=8)   # r = 76, 512-byte rows
    check_case(ctx, make_case(w, gain=4.0))


def test_many_pairs_small_heads(ctx):
    w = wl.shrink(wl.WORKLOADS[2], B=24, H=64, d=16, N=520, n_cal=64, heavy_count=6)   # 1536 pairs, r = 4
    check_case(ctx, make_case(w, gain=2.0))


@pytest.mark.parametrize("cfg,B,H,N,gain", [
    (4, 20, 7, 600, 10.0),     # 20 sequences: projection with the x fragments shared through LDS; 17 column blocks
    (3, 18, 3, 700, 16.0),     # the same for a rotary model (every column of W_q)
    (4, 32, 6, 300, 10.0),     # both batch blocks full
])
def test_seventeen_to_thirty_two_sequences(ctx, cfg, B, H, N, gain):
    w = wl.shrink(wl.WORKLOADS[cfg], B=B, H=H, N=N, n_cal=256, heavy_count=8, pool="hbm")
    check_case(ctx, make_case(w, gain=gain))


def test_cfg3_shape_rope_f16(ctx):
    w = wl.shrink(wl.WORKLOADS[3], B=2, H=4, N=4096)
    check_case(ctx, make_case(w, gain=24.0))


def test_cfg3_shape_rope_with_bias_ragged(ctx):
    w = wl.shrink(wl.WORKLOADS[3], B=3, H=2, N=1234)
    check_case(ctx, make_case(w, gain=16.0, bias=True, N_cap=1500))


@pytest.mark.parametrize("cfg,B,H,d,N,N_cap,gain,bias", [
    (2, 8, 8, 32, 9000, 9000, 6.0, False),       # 18 tiles of 512: two passes of the 16 waves, ragged tail
    (3, 4, 16, 32, 12345, 13000, 20.0, True),    # rotary, spare capacity, bias
    (5, 2, 32, 16, 32768, 32768, 40.0, False),   # the longest sequence this path takes (64 tiles), rotary
    (1, 8, 8, 32, 5000, 5100, 8.0, False),       # float32: tiles of 256 tokens, 20 of them
    (2, 8, 8, 32, 9000, 40000, 6.0, False),      # capacity far beyond the valid tokens: only 18 of 79 tiles are read
])
def test_long_sequences_many_pairs_scores_parked_in_lds(ctx, cfg, B, H, d, N, N_cap, gain, bias):
    w = wl.shrink(wl.WORKLOADS[cfg], B=B, H=H, d=d, N=N, n_cal=max(64, 2 * d), heavy_count=24)
    check_case(ctx, make_case(w, gain=gain, bias=bias, N_cap=N_cap), host_pool=False)


def test_cfg5_shape_long_context_tiled_path(ctx):
    w = wl.shrink(wl.WORKLOADS[5], B=1, H=2, N=20000)
    check_case(ctx, make_case(w, gain=6.0, N_cap=20480))


@pytest.mark.parametrize("B,H,N", [
    (8, 8, 8192),     # 16 tiles: the last shape of the 16-wave register form
    (8, 8, 8193),     # 17 tiles, 64 pairs: scores parked in LDS
    (7, 9, 8193),     # 63 pairs: too few for one workgroup per pair, one wave per tile
    (4, 16, 32769),   # 65 tiles: beyond the LDS form
])
def test_scan_form_boundaries(ctx, B, H, N):
    w = wl.shrink(wl.WORKLOADS[2], B=B, H=H, d=16, N=N, ratio=0.5, n_cal=64, heavy_count=12)
    check_case(ctx, make_case(w, gain=8.0))


def test_long_sequence_tiled_path_with_spare_capacity(ctx):
    w = wl.shrink(wl.WORKLOADS[5], B=1, H=2, N=9000)              # 18 valid tiles of 98 allocated
    check_case(ctx, make_case(w, gain=6.0, N_cap=50000))


def test_f32_long_sequence_tiled_path(ctx):
    w = wl.shrink(wl.WORKLOADS[1], B=1, H=2, N=5000, heavy_count=16)
    check_case(ctx, make_case(w, gain=8.0))


@pytest.mark.parametrize("B", [20, 40])
def test_projection_with_more_than_sixteen_sequences(ctx, B):
    w = wl.shrink(wl.WORKLOADS[4], B=B, H=2, N=600, pool="hbm")
    check_case(ctx, make_case(w, gain=6.0))


def test_f16_model_dimension_not_multiple_of_32_uses_fma_projection(ctx):
    w = wl.shrink(wl.WORKLOADS[2], B=2, H=3, d=8, N=900, ratio=0.5, n_cal=64, heavy_count=5)
    check_case(ctx, make_case(w, gain=2.0))


def _random_shapes():
    rng = np.random.default_rng(20240627)
    cases = []
    for i in range(14):
        f16 = bool(rng.integers(0, 2))
        rope = bool(rng.integers(0, 2))
        d = int(rng.choice([8, 16, 32, 64, 128] if f16 else [4, 8, 16, 32, 64]))
        if rope and d % 2:
            d *= 2
        H = int(rng.integers(1, 7))
        B = int(rng.integers(1, 6))
        N = int(rng.integers(1, 2600))
        N_cap = N + int(rng.integers(0, 3)) * int(rng.integers(1, 300))
        ratio = float(rng.choice([0.2, 0.3, 0.5, 0.75, 1.0]))
        if int(ratio * d) < 1:
            ratio = 1.0
        cases.append(pytest.param(dict(B=B, H=H, d=d, N=N, dtype="f16" if f16 else "f32", rope=rope,
                                       ratio=ratio, n_cal=64, heavy_count=min(5, N)),
                                  N_cap, float(rng.choice([1.0, 3.0, 8.0])), bool(rng.integers(0, 2)),
                                  id=f"r{i}-B{B}H{H}d{d}N{N}"))
    return cases


def _random_long_shapes():
    # many pairs and long sequences: random draws around the switches between the scan's forms
    # (16-wave registers / LDS-parked scores / one wave per tile; 64 pairs; 32768 tokens)
    rng = np.random.default_rng(19707)
    cases = []
    for i in range(8):
        f16 = bool(rng.integers(0, 2))
        rope = bool(rng.integers(0, 2))
        d = int(rng.choice([8, 16, 32]))
        B = int(rng.integers(2, 12))
        H = int(rng.integers(4, 17))
        tile = 512 if f16 else 256
        N = int(rng.integers(12 * tile, 40 * tile if f16 else 70 * tile))
        N_cap = N + int(rng.integers(0, 2)) * int(rng.integers(1, 3000))
        ratio = float(rng.choice([0.3, 0.5, 1.0]))
        cases.append(pytest.param(dict(B=B, H=H, d=d, N=N, dtype="f16" if f16 else "f32", rope=rope,
                                       ratio=ratio, n_cal=64, heavy_count=16),
                                  N_cap, float(rng.choice([4.0, 8.0, 16.0])), bool(rng.integers(0, 2)),
                                  id=f"l{i}-B{B}H{H}d{d}N{N}-{'f16' if f16 else 'f32'}"))
    return cases


@pytest.mark.parametrize("shape,N_cap,gain,bias", _random_shapes() + _random_long_shapes())
def test_seeded_random_shapes(ctx, shape, N_cap, gain, bias):
    w = wl.shrink(wl.WORKLOADS[2], **shape)
    check_case(ctx, make_case(w, gain=gain, N_cap=N_cap, bias=bias))


def test_host_pinned_pool_gather(ctx):
    w = wl.shrink(wl.WORKLOADS[4], B=2, H=4, N=2048)
    check_case(ctx, make_case(w, gain=6.0), host_pool=True)


def test_list_longer_than_stride_is_clamped_and_flagged(ctx):
    import paper_2406_19707_amd as ig
    from ig_gpu import run_gpu
    w = wl.shrink(wl.WORKLOADS[2], B=2, H=2, N=1024)
    c = make_case(w, gain=1.0)                       # literal scale: every token selected
    got = run_gpu(ctx, c, sel_stride=100)
    assert got["status"] == ig.IG_ECAPACITY
    assert np.all(got["sel_cnt"] == 100)
    assert np.array_equal(got["sel_idx"], np.tile(np.arange(100, dtype=np.int32), (4, 1)))
    assert ctx.ig_check_status() == ig.IG_OK          # the flag is cleared by the check


def test_selection_is_deterministic(ctx):
    from ig_gpu import run_gpu, Uploaded
    w = wl.shrink(wl.WORKLOADS[2], B=4, H=8, N=2048)
    c = make_case(w, gain=5.0)
    up = Uploaded(ctx, c)
    first = run_gpu(ctx, c, up=up)
    for _ in range(19):
        again = run_gpu(ctx, c, up=up)
        assert np.array_equal(again["sel_cnt"], first["sel_cnt"])
        assert np.array_equal(again["sel_idx"], first["sel_idx"])
        assert np.array_equal(again["out"], first["out"])


def test_empty_list_without_new_row_gives_zeros(ctx):
    import paper_2406_19707_amd as ig
    from ig_gpu import desc_of, dev
    w = wl.shrink(wl.WORKLOADS[2], B=1, H=2, N=64)
    c = make_case(w)
    d = desc_of(c)
    cnt = torch.zeros(2, dtype=torch.int32, device="cuda")
    Ks = torch.ones((2, 64, w.d), dtype=torch.float16, device="cuda")
    out = torch.full((1, 2, w.d), float("nan"), dtype=torch.float16, device="cuda")
    ctx.ig_sparse_attention(d, dev(c.q), Ks, Ks, cnt, 64, None, None, out)
    assert torch.all(out == 0)
    kn, vn = dev(c.k_new), dev(c.v_new)
    ctx.ig_sparse_attention(d, dev(c.q), Ks, Ks, cnt, 64, kn, vn, out)
    assert torch.allclose(out, vn, atol=1e-3)         # only the new row: weight 1


def test_error_paths(ctx):
    import ctypes
    import paper_2406_19707_amd as ig
    w = wl.shrink(wl.WORKLOADS[2], B=1, H=2, N=64)
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    p = buf.data_ptr()

    def spec(desc, **kw):
        a = dict(x=p, wq=p, slab=p, sel_idx=p, stride=64, cnt=p)
        a.update(kw)
        return ctx.call("ig_speculate", ctypes.byref(desc), a["x"], a["wq"], None, None, None,
                        a["slab"], a["sel_idx"], a["stride"], a["cnt"], None, 0)

    good = dict(B=1, H=2, d=128, r=38, N=64)
    assert spec(ig.IgDesc(**good, alpha=-1.0)) == ig.IG_EINVAL
    assert "alpha" in ctx.last_error()
    assert spec(ig.IgDesc(**good, alpha=float("nan"))) == ig.IG_EINVAL
    assert spec(ig.IgDesc(B=1, H=2, d=128, r=200, N=64)) == ig.IG_ESHAPE
    assert spec(ig.IgDesc(B=1, H=2, d=128, r=38, N=0)) == ig.IG_ESHAPE
    assert spec(ig.IgDesc(B=1, H=2, d=128, r=38, N=64, N_cap=32)) == ig.IG_ESHAPE
    assert spec(ig.IgDesc(**good, dtype=9)) == ig.IG_EDTYPE
    assert spec(ig.IgDesc(B=1, H=2, d=4, r=2, N=64)) == ig.IG_ESHAPE      # 8-byte rows
    assert spec(ig.IgDesc(**good), x=None) == ig.IG_EINVAL
    assert spec(ig.IgDesc(**good), stride=0) == ig.IG_ESHAPE
    assert spec(ig.IgDesc(**good, rope=1)) == ig.IG_EINVAL                 # rope without A_p / pos
    # a pageable host buffer passed as a pinned pool is refused
    d = ig.IgDesc(**good)
    host = np.zeros(1 << 16, np.uint8)
    rc = ctx.call("ig_gather_kv", ctypes.byref(d), host.ctypes.data, host.ctypes.data,
                  ig.IG_MEM_HOST_PINNED, p, 64, p, p, p, 0)
    assert rc == ig.IG_EINVAL and "pinned" in ctx.last_error()
    rc = ctx.call("ig_gather_kv", ctypes.byref(d), p, p, 7, p, 64, p, p, p, 0)
    assert rc == ig.IG_EINVAL
    torch.cuda.synchronize()
