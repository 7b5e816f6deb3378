"""GPU parity of nova_merge_cache_interp (nearest-cell and cubic-convolution interpolation of the residual
cache, Sec. 3.3 "Residual Cache Reuse": the cache is interpolated to the next scale's grid) against the
oracle.  Nearest is a copy: exact.  Bicubic: fp32 taps, one rounding to the storage type."""
import numpy as np
import pytest
import torch

import workloads as WL
from oracle import nova_oracle as O

pytestmark = pytest.mark.gpu

INTERP = {"bilinear": 0, "nearest": 1, "bicubic": 2}


@pytest.fixture(scope="module")
def hx():
    import harness
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU and the built libnova.so (no fallback)")
    return harness


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("interp", ["nearest", "bicubic", "bilinear"])
@pytest.mark.parametrize("grids", [((13, 13), (16, 16)), ((3, 5), (7, 6)), ((16, 16), (16, 16)), ((48, 48), (64, 64)),
                                   ((5, 5), (4, 4)), ((1, 1), (3, 2)), ((6, 4), (12, 12))])
def test_merge_interp_matches_oracle(hx, dtype, interp, grids):
    (hp, wp), (h, w) = grids
    print(f"merge {interp} dtype={dtype} {hp}x{wp}->{h}x{w}", flush=True)
    td = WL.torch_dtype(dtype)
    g = torch.Generator().manual_seed(hp * 1000 + wp * 100 + h * 10 + w)
    B, C, N = 2, 72 if dtype == "f32" else 136, h * w
    x = torch.randn((B, N, C), generator=g).to(td)
    prev = torch.randn((B, hp * wp, C), generator=g).to(td)
    for k in sorted({0, 1, N // 2, N}):
        H = torch.rand((B, N), generator=g).numpy()
        idx, mask = O.select(H, k)
        y = torch.randn((B, max(k, 1), C), generator=g).to(td)
        out = torch.empty((B, N, C), dtype=td, device="cuda")
        cn = torch.empty((B, N, C), dtype=td, device="cuda")
        cache = prev.cuda() if k < N else torch.full_like(prev, float("nan")).cuda()
        hx.nova().merge_cache_interp(INTERP[interp], h, w, hp, wp, k, x.cuda(), y.cuda(),
                                     torch.from_numpy(idx if k else np.zeros((B, 1), np.int32)).cuda(),
                                     torch.from_numpy(mask).cuda(), cache, out, cn)
        torch.cuda.synchronize()
        ro, rc = O.merge_cache(hx.f64(x), hx.f64(y)[:, :k], idx[:, :k], hx.f64(prev), hp, wp, h, w, interp=interp)
        if interp == "nearest":
            # cache_new of a pruned row is a copy of a stored cache row; out = x + that row, rounded once
            pruned = mask == 0
            assert np.array_equal(hx.f64(cn)[pruned], rc[pruned])
            ref_out = torch.from_numpy(ro).to(td).to(torch.float64).numpy()
            assert np.array_equal(hx.f64(out)[pruned], ref_out[pruned])
        tol = hx.BF16_TOL if dtype == "bf16" else 2e-6
        assert hx.nerr(out, ro) <= tol and hx.nerr(cn, rc, scale_ref=ro) <= tol
        for b in range(B):                                  # kept rows are copied bit for bit
            if k:
                assert torch.equal(out[b, torch.from_numpy(idx[b, :k]).long().cuda()].cpu(), y[b, :k])


def test_bilinear_through_the_interp_entry_point_is_nova_merge_cache(hx):
    g = torch.Generator().manual_seed(3)
    B, C, hp, h = 2, 128, 9, 12
    N, k = h * h, 50
    x = torch.randn((B, N, C), generator=g).to(torch.bfloat16).cuda()
    prev = torch.randn((B, hp * hp, C), generator=g).to(torch.bfloat16).cuda()
    y = torch.randn((B, k, C), generator=g).to(torch.bfloat16).cuda()
    idx, mask = O.select(torch.rand((B, N), generator=g).numpy(), k)
    idx, mask = torch.from_numpy(idx).cuda(), torch.from_numpy(mask).cuda()
    res = []
    for call in ("plain", "interp"):
        out = torch.empty_like(x); cn = torch.empty_like(x)
        if call == "plain":
            hx.nova().merge_cache(h, h, hp, hp, k, x, y, idx, mask, prev, out, cn)
        else:
            hx.nova().merge_cache_interp(0, h, h, hp, hp, k, x, y, idx, mask, prev, out, cn)
        torch.cuda.synchronize()
        res.append((out, cn))
    assert torch.equal(res[0][0], res[1][0]) and torch.equal(res[0][1], res[1][1])


def test_interp_argument_errors(hx):
    from paper_2602_01345_amd import NovaError
    x = torch.zeros((1, 4, 8), dtype=torch.float32, device="cuda")
    out = torch.full_like(x, 5.0)
    mask = torch.zeros((1, 4), dtype=torch.uint8, device="cuda")
    prev = torch.zeros((1, 1, 8), dtype=torch.float32, device="cuda")
    for bad in (-1, 3, 99):
        with pytest.raises(NovaError) as e:
            hx.nova().merge_cache_interp(bad, 2, 2, 1, 1, 0, x, None, None, mask, prev, out, None)
        assert e.value.code == -1
    torch.cuda.synchronize()
    assert bool((out == 5.0).all())
