"""GPU parity of the prefill-side partial weight index (ig_partial_index_device) against the
oracle's column ranking (Section 4.3 "Prefill Stage").  The GPU sums in float32, the oracle in
double: the kept sets must agree except for columns whose oracle sums lie within 1e-5 (relative)
of the r-th largest sum."""
import numpy as np
import pytest
import torch

from oracle import ig_oracle as o

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_2406_19707_amd as ig
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = ig.Context(0)
    yield c
    c.close()


@pytest.mark.parametrize("H,d,n,ratio,dtype,with_keys", [
    (32, 128, 2048, 0.3, "f16", True),
    (4, 64, 512, 0.3, "f32", False),
    (5, 96, 333, 0.2, "f16", True),      # ragged rows / columns
    (2, 256, 40, 0.5, "f32", True),
    (3, 8, 7, 0.3, "f32", False),        # fewer rows than row chunks
])
def test_kept_columns_match_the_oracle(ctx, H, d, n, ratio, dtype, with_keys):
    import paper_2406_19707_amd as ig
    print(f"case H{H} d{d} n{n} ratio {ratio} {dtype} keys {with_keys}", flush=True)
    rng = np.random.default_rng(H * 1000 + d + n)
    npdt = np.float16 if dtype == "f16" else np.float32
    col_gain = rng.uniform(0.2, 3.0, (1, H * d))
    Qs = (rng.standard_normal((n, H * d)) * col_gain).astype(npdt)
    Ks = (rng.standard_normal((n, H * d)) * col_gain[:, ::-1]).astype(npdt) if with_keys else None
    ref = o.partial_index(Qs.astype(np.float32), None if Ks is None else Ks.astype(np.float32), H, ratio)
    r = ref.shape[1]
    idx = torch.full((H, r), -1, dtype=torch.int32, device="cuda")
    q_dev = torch.from_numpy(Qs).cuda()
    k_dev = None if Ks is None else torch.from_numpy(Ks).cuda()
    code = ig.IG_F16 if dtype == "f16" else ig.IG_F32
    ctx.ig_partial_index_device(code, H, d, n, q_dev, k_dev, ratio, idx)
    torch.cuda.synchronize()
    got = idx.cpu().numpy()
    again = torch.full_like(idx, -1)
    ctx.ig_partial_index_device(code, H, d, n, q_dev, k_dev, ratio, again)
    torch.cuda.synchronize()
    assert torch.equal(idx, again)                               # repeatable bit for bit
    sums = np.abs(Qs.astype(np.float64)).sum(0) + (0 if Ks is None else np.abs(Ks.astype(np.float64)).sum(0))
    for h in range(H):
        assert np.all(np.diff(got[h]) > 0) and got[h][0] >= 0 and got[h][-1] < d
        diff = np.setxor1d(got[h], ref[h])
        if diff.size:
            c = sums[h * d:(h + 1) * d]
            cut = np.sort(c)[::-1][r - 1]
            assert np.all(np.abs(c[diff] - cut) <= 1e-5 * cut), (h, diff)


def test_equal_sums_keep_the_lower_columns(ctx):
    import paper_2406_19707_amd as ig
    Qs = torch.ones((16, 2 * 64), dtype=torch.float32, device="cuda")
    idx = torch.zeros((2, 19), dtype=torch.int32, device="cuda")
    ctx.ig_partial_index_device(ig.IG_F32, 2, 64, 16, Qs, None, 0.3, idx)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), np.tile(np.arange(19, dtype=np.int32), (2, 1)))


def test_error_paths(ctx):
    import paper_2406_19707_amd as ig
    buf = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    p = buf.data_ptr()
    call = lambda *a: ctx.call("ig_partial_index_device", *a)  # noqa: E731
    assert call(ig.IG_F32, 2, 300, 4, p, None, 0.3, p, 0) == ig.IG_ESHAPE       # d > 256
    assert call(9, 2, 64, 4, p, None, 0.3, p, 0) == ig.IG_EDTYPE
    assert call(ig.IG_F32, 2, 64, 4, None, None, 0.3, p, 0) == ig.IG_EINVAL
    assert call(ig.IG_F32, 2, 64, 4, p, None, 0.0, p, 0) == ig.IG_EINVAL
    assert call(ig.IG_F32, 2, 2, 4, p, None, 0.3, p, 0) == ig.IG_ESHAPE         # floor(0.3 * 2) = 0
