"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Tolerances: kept-index lists and masks bit-exact; fp32 entropies |dH| <= 1e-5|H| + 1e-7;
bf16 tensors max|d|/max|ref| <= 2e-2; fp32 block tensors <= 2e-5 (fp32 accumulation over
at most 256 terms).  Selection is always compared on the same fp32 entropy array.
"""
import math

import numpy as np
import pytest
import torch

import workloads as WL
from oracle import nova_oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hx():
    import harness
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU and the built libnova.so (no fallback)")
    return harness


def _say(msg):
    print(msg, flush=True)


# ----------------------------------------------------------------------------------
# entropy
# ----------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V", [512, 4096, 1000, 513, 7, 1, 20000])
def test_entropy_matches_oracle(hx, dtype, V):
    _say(f"entropy dtype={dtype} V={V}")
    wl = WL.Workload("t", dtype, B=3, C=64, heads=4, L=1, V=V, keep_hi=.5, keep_lo=.5,
                     scales=(WL.Scale(grid=9, prev_grid=7, kv_len=10),), seed=3)
    logits = WL.make_logits(wl, 0)                       # [3, 81, V] log-uniform temperatures
    d = logits.cuda()
    H = torch.empty((3, 81), dtype=torch.float32, device="cuda")
    mean = torch.empty((3,), dtype=torch.float32, device="cuda")
    hx.nova().entropy(d, H, mean)
    torch.cuda.synchronize()
    ref = O.entropy(hx.f64(logits))
    assert hx.entropy_ok(H, ref)
    assert np.allclose(mean.cpu().numpy(), O.mean_entropy(ref), rtol=2e-5, atol=1e-6)


def test_entropy_closed_forms_and_edge_rows(hx):
    _say("entropy closed forms")
    V = 4096
    x = torch.zeros((1, 8, V), dtype=torch.float32)
    x[0, 0] = 3.25                                      # uniform -> ln V
    x[0, 1] = -1e4; x[0, 1, 77] = 50.0                  # one-hot -> 0
    x[0, 2, :16] = 3.0                                  # two-level
    x[0, 3] = torch.linspace(-30, 30, V)
    x[0, 4] = float("-inf"); x[0, 4, 5] = 1.0; x[0, 4, 9] = 1.0   # two survivors -> ln 2
    x[0, 5, 100] = float("nan")                         # NaN row -> NaN
    x[0, 6] = 1e4 + torch.randn(V, generator=torch.Generator().manual_seed(0))   # huge offset
    x[0, 7, 0] = 20.0                                   # tiny entropy
    H = torch.empty((1, 8), dtype=torch.float32, device="cuda")
    hx.nova().entropy(x.cuda(), H)
    got = H.cpu().numpy()[0]
    assert got[0] == pytest.approx(math.log(V), rel=1e-6)
    assert got[1] == 0.0
    assert got[4] == pytest.approx(math.log(2.0), rel=1e-6)
    assert math.isnan(got[5])
    ref = O.entropy(hx.f64(x))[0]
    ok = [0, 1, 2, 3, 4, 6, 7]
    assert hx.entropy_ok(got[ok], ref[ok])
    assert got[7] == pytest.approx(0.00017724744533827648, rel=1e-5)


def test_entropy_strided_and_unaligned_rows(hx):
    _say("entropy strided/unaligned")
    g = torch.Generator().manual_seed(1)
    base = (torch.randn((2, 50, 1030), generator=g) * 4).to(torch.bfloat16).cuda()
    view = base[:, :, :1001]                            # row stride 1030, V = 1001: rows not 16-byte aligned
    H = torch.empty((2, 50), dtype=torch.float32, device="cuda")
    n = hx.nova()
    rc = n.lib.nova_entropy(n.ctx, None, view.data_ptr(), 1, 50, 2, 1001, 1030, H.data_ptr(), None)
    assert rc == 0
    torch.cuda.synchronize()
    assert hx.entropy_ok(H, O.entropy(hx.f64(view)))


# ----------------------------------------------------------------------------------
# selection
# ----------------------------------------------------------------------------------
def _run_select(hx, H32, k, k_per_row=None):
    B, N = H32.shape
    d = torch.from_numpy(H32).cuda()
    idx = torch.full((B, max(k, 1)), -7, dtype=torch.int32, device="cuda")
    mask = torch.full((B, N), 9, dtype=torch.uint8, device="cuda")
    kp = None if k_per_row is None else torch.tensor(k_per_row, dtype=torch.int32, device="cuda")
    hx.nova().select(d, k, idx, mask, kp)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), mask.cpu().numpy()


@pytest.mark.parametrize("N", [1, 63, 169, 256, 1024, 4096, 5000, 8192, 8193, 16384, 40000])
def test_select_bit_exact(hx, N):
    _say(f"select N={N}")
    rng = np.random.default_rng(N)
    H = (rng.random((3, N)) * 8.3).astype(np.float32)
    H[1] = np.round(H[1] * 4) / 4                      # heavy ties
    H[2, ::7] = 0.0
    H[2, 1::13] = -0.0
    if N > 20:
        H[2, 5] = np.nan
        H[2, 11] = np.inf
    for k in sorted({0, 1, N // 3, N // 2, N - 1, N}):
        if k < 0:
            continue
        idx, mask = _run_select(hx, H, k)
        ridx, rmask = O.select(H, k)
        assert np.array_equal(mask, rmask), f"mask differs at k={k}"
        assert np.array_equal(idx[:, :k], ridx[:, :k]), f"idx differs at k={k}"


def test_select_all_equal_and_per_row_k(hx):
    _say("select all-equal / per-row k")
    H = np.full((4, 777), 1.5, dtype=np.float32)
    idx, mask = _run_select(hx, H, 100)
    assert np.array_equal(idx, np.tile(np.arange(100, dtype=np.int32), (4, 1)))
    rng = np.random.default_rng(0)
    H = rng.random((4, 300)).astype(np.float32)
    ks = [0, 17, 300, 120]
    idx, mask = _run_select(hx, H, 300, ks)
    ridx, rmask = O.select(H, ks)
    assert np.array_equal(mask, rmask)
    assert np.array_equal(idx, ridx)                    # including the -1 tails


# ----------------------------------------------------------------------------------
# merge
# ----------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("grids", [(13, 16), (3, 7), (16, 16), (48, 64), (5, 4)])
def test_merge_matches_oracle(hx, dtype, grids):
    hp, h = grids
    _say(f"merge dtype={dtype} {hp}->{h}")
    td = WL.torch_dtype(dtype)
    tol = hx.BF16_TOL if dtype == "bf16" else 1e-6
    g = torch.Generator().manual_seed(hp * 100 + h)
    B, C, N = 2, 72 if dtype == "f32" else 136, h * h
    x = torch.randn((B, N, C), generator=g).to(td)
    prev = torch.randn((B, hp * hp, C), generator=g).to(td)
    for k in sorted({0, 1, N // 2, N}):
        H = torch.rand((B, N), generator=g).numpy()
        idx, mask = O.select(H, k)
        y = torch.randn((B, max(k, 1), C), generator=g).to(td)
        out = torch.empty((B, N, C), dtype=td, device="cuda")
        cn = torch.empty((B, N, C), dtype=td, device="cuda")
        cache = prev.cuda() if k < N else torch.full_like(prev, float("nan")).cuda()
        hx.nova().merge_cache(h, h, hp, hp, k, x.cuda(), y.cuda(),
                              torch.from_numpy(idx if k else np.zeros((B, 1), np.int32)).cuda(),
                              torch.from_numpy(mask).cuda(), cache, out, cn)
        torch.cuda.synchronize()
        ro, rc = O.merge_cache(hx.f64(x), hx.f64(y)[:, :k], idx[:, :k], hx.f64(prev), hp, hp, h, h)
        assert hx.nerr(out, ro) <= tol and hx.nerr(cn, rc) <= tol
        # kept rows are copied bit for bit
        for b in range(B):
            if k:
                assert torch.equal(out[b, torch.from_numpy(idx[b, :k]).long().cuda()].cpu(), y[b, :k])
    # no prior cache at all when every token is kept
    hx.nova().merge_cache(h, h, hp, hp, N, x.cuda(), y.cuda(), torch.from_numpy(idx).cuda(),
                          torch.from_numpy(mask).cuda(), None, out, None)
    torch.cuda.synchronize()
    assert torch.equal(out.cpu(), y)


# ----------------------------------------------------------------------------------
# the block, small shapes spanning several tiles with ragged tails
# ----------------------------------------------------------------------------------
def _custom(dtype, B, grid, prev, P, C, heads, V=64, seed=5):
    return WL.Workload("custom", dtype, B=B, C=C, heads=heads, L=1, V=V, keep_hi=.5, keep_lo=.5,
                       scales=(WL.Scale(grid=grid, prev_grid=prev, kv_len=P),), seed=seed)


@pytest.mark.parametrize("C,heads", [(128, 2), (256, 2), (192, 3)])
@pytest.mark.parametrize("k", [1, 150, 289])
def test_block_bf16_small(hx, C, heads, k):
    _say(f"block bf16 C={C} heads={heads} k={k}")
    wl = _custom("bf16", B=2, grid=17, prev=13, P=100, C=C, heads=heads)
    hb = hx.make_host_block(wl, 0, k=k)
    errs = hx.check_block(hb, hx.BF16_TOL)
    _say(f"   errors {errs}")


@pytest.mark.parametrize("k", [0, 1, 37, 100])
def test_block_f32_small(hx, k):
    _say(f"block f32 k={k}")
    wl = _custom("f32", B=2, grid=10, prev=7, P=45, C=48, heads=3)
    hb = hx.make_host_block(wl, 0, k=k)
    errs = hx.check_block(hb, hx.F32_TOL)
    _say(f"   errors {errs}")


def test_block_f32_rows_wider_than_the_layer_norm_register_path(hx):
    """C = 2304 in fp32 is 576 16-byte vectors per row, more than a wave of the LayerNorm kernel keeps in
    registers: the rows go through its three-pass form."""
    _say("block f32 C=2304 k=3")
    wl = _custom("f32", B=1, grid=4, prev=3, P=8, C=2304, heads=36)
    errs = hx.check_block(hx.make_host_block(wl, 0, k=3), hx.F32_TOL)
    _say(f"   errors {errs}")


@pytest.mark.parametrize("k", [1, 40, 100])
def test_block_bf16_few_rows_long_ffn(hx, k):
    """Few kept rows and an FFN hidden width of 4096: the down projection sums K in slices over several
    workgroups and a second pass adds the slices (M = 2, 80, 200 rows)."""
    _say(f"block bf16 C=1024 F=4096 k={k}")
    wl = _custom("bf16", B=2, grid=10, prev=7, P=64, C=1024, heads=8)
    errs = hx.check_block(hx.make_host_block(wl, 0, k=k), hx.BF16_TOL)
    _say(f"   errors {errs}")


def test_block_keep_zero_bf16(hx):
    _say("block bf16 k=0")
    wl = _custom("bf16", B=2, grid=8, prev=6, P=64, C=128, heads=2)
    hx.check_block(hx.make_host_block(wl, 0, k=0), hx.BF16_TOL)


# ----------------------------------------------------------------------------------
# the five workloads (first and last block of the last scale; a subset of batch rows where
# the oracle would take too long)
# ----------------------------------------------------------------------------------
def test_cfg1_full_step(hx):
    _say("cfg1 full")
    wl = WL.WORKLOADS["cfg1"]
    errs = hx.check_block(hx.make_host_block(wl, 0), hx.F32_TOL)
    _say(f"   errors {errs}")


@pytest.mark.parametrize("name,rows", [("cfg2", None), ("cfg3", [0, 15]), ("cfg4", [3]), ("cfg5", [1])])
@pytest.mark.parametrize("which", ["first", "last"])
def test_workload_blocks(hx, name, rows, which):
    wl = WL.WORKLOADS[name]
    j = 0 if which == "first" else wl.L - 1
    _say(f"{name} block {j} k={wl.k(j)} rows={rows}")
    errs = hx.check_block(hx.make_host_block(wl, j), hx.BF16_TOL, rows=rows)
    _say(f"   errors {errs}")


@pytest.mark.parametrize("j", [21, 27])
def test_cfg5_middle_blocks_ragged_last_rounds(hx, j):
    """cfg5 block 22 (k = 1348): 352 attention items for 512 workgroup slots, the case in which one uncut item
    per CU runs next to items cut into key runs.  Block 28 (k = 1031, 2062 rows): the projections cover 2048 rows
    with one whole round of large tiles and the last 14 rows with the narrow-tile kernels (K-sliced for the FFN
    down projection)."""
    wl = WL.WORKLOADS["cfg5"]
    _say(f"cfg5 block {j} k={wl.k(j)}")
    errs = hx.check_block(hx.make_host_block(wl, j), hx.BF16_TOL, rows=[0])
    _say(f"   errors {errs}")


@pytest.mark.parametrize("name,blocks,row", [("cfg5", (4, 8, 12, 16, 20, 24), 1), ("cfg4", (9, 18, 27), 6),
                                             ("cfg3", (7, 15, 22), 9), ("cfg2", (3, 5, 8, 11, 13), 4)])
def test_workload_blocks_in_between(hx, name, blocks, row):
    """More blocks of every workload's last scale, one image each: the keep count (and with it every launch plan:
    tile shapes, two-launch row plans, K slices, attention key runs) changes from block to block."""
    wl = WL.WORKLOADS[name]
    for j in blocks:
        _say(f"{name} block {j} k={wl.k(j)} row {row}")
        errs = hx.check_block(hx.make_host_block(wl, j), hx.BF16_TOL, rows=[row])
        _say(f"   errors {errs}")


@pytest.mark.parametrize("name,si,rows", [("cfg3", 0, [1]), ("cfg4", 0, [2]), ("cfg4", 1, [5]), ("cfg5", 0, [0]),
                                          ("cfg5", 1, [1]), ("cfg5", 2, [0])])
def test_earlier_pruned_scales(hx, name, si, rows):
    """Every pruned scale before the last one: cfg3 at 13x13 (prior grid 10), cfg4 at 18x18 and 24x24 (prior grids
    13 and 18, P = 316 and 640), cfg5 at 32x32, 40x40 and 48x48 (prior grids 24, 32, 40; P = 1497, 2521, 4121):
    other upsampling ratios, attention split plans and GEMM row plans than the last scale's.  Block 1, one image."""
    wl = WL.WORKLOADS[name]
    s = wl.scales[si]
    assert s is not wl.last
    _say(f"{name} scale {s.grid}x{s.grid} prior grid {s.prev_grid} P={s.kv_len} k={wl.k(1, s)} rows={rows}")
    errs = hx.check_block(hx.make_host_block(wl, 1, scale=s), hx.BF16_TOL, rows=rows)
    _say(f"   errors {errs}")


def test_cache_new_error_on_its_own_scale_is_on_record(hx):
    """The new residual cache is out - x, a difference of two stored bf16 tensors, so its error is checked on the
    scale of `out`.  This prints the same error on the residual's own scale with half of the tokens kept and with
    every token kept (then the residual is only the block's update, much smaller than the activations)."""
    wl = _custom("bf16", B=2, grid=17, prev=13, P=300, C=256, heads=2)
    for k in (144, 289):
        errs = hx.check_block(hx.make_host_block(wl, 0, k=k), hx.BF16_TOL)
        _say(f"   k={k} of 289: cache_new error / max|out| = {errs['cache_new']:.3e}, "
             f"/ max|cache_new| = {errs['cache_new_own_scale']:.3e}")
        assert errs["cache_new_own_scale"] >= errs["cache_new"] * 0.999


# ----------------------------------------------------------------------------------
# argument errors are reported, not launched
# ----------------------------------------------------------------------------------
def test_argument_errors(hx):
    _say("argument errors")
    n = hx.nova()
    H = torch.zeros((2, 16), dtype=torch.float32, device="cuda")
    idx = torch.zeros((2, 16), dtype=torch.int32, device="cuda")
    mask = torch.zeros((2, 16), dtype=torch.uint8, device="cuda")
    lib = n.lib
    assert lib.nova_select(n.ctx, None, H.data_ptr(), 2, 16, 17, None, idx.data_ptr(), mask.data_ptr()) == -1
    assert lib.nova_select(n.ctx, None, None, 2, 16, 4, None, idx.data_ptr(), mask.data_ptr()) == -1
    assert lib.nova_select(n.ctx, None, H.data_ptr(), 2, 70000, 4, None, idx.data_ptr(), mask.data_ptr()) == -2
    assert lib.nova_entropy(n.ctx, None, H.data_ptr(), 0, 16, 2, 0, 0, H.data_ptr(), None) == -1
    assert lib.nova_entropy(n.ctx, None, H.data_ptr(), 5, 16, 2, 1, 1, H.data_ptr(), None) == -2
    from paper_2602_01345_amd import BlockShape
    bad = BlockShape(1, 2, 16, 128, 3, 0, 64, 4)          # C % heads != 0
    assert n.workspace_bytes(bad) == 0
    ok = BlockShape(1, 2, 16, 128, 2, 0, 64, 4)
    assert n.workspace_bytes(ok) > 0
    assert n.workspace_bytes(BlockShape(1, 2, 16, 128, 2, 62, 64, 4)) == 0     # P + k > capacity
    assert n.workspace_bytes(BlockShape(1, 2, 16, 96, 2, 0, 64, 4)) == 0       # dh = 48 unsupported in bf16


def test_probe_kernels_report_their_work(hx):
    """The achievable-peak probes (instrumentation) run and report bytes / flops; the copy copies."""
    nova = hx.nova()
    sink = torch.zeros(1, device="cuda")
    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    assert nova.probe(0, src, None, 1, sink) == src.numel() * 4
    assert nova.probe(1, src, dst, 1, sink) == 2 * src.numel() * 4
    flops = nova.probe(2, None, None, 3, sink)
    torch.cuda.synchronize()
    assert torch.equal(src, dst) and float(sink) == 0.0
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert flops == cus * 8 * 3 * 32 * 2 * 32 * 32 * 16
    # the same loop on operands read from memory: needs 128 bytes per lane of CUs x 512 lanes
    data = torch.randn(cus * 512 * 64, device="cuda").to(torch.bfloat16)
    assert nova.probe(3, data, None, 3, sink) == flops
    with pytest.raises(Exception):
        nova.probe(3, data[: data.numel() // 2], None, 3, sink)        # too few operands: rejected before the launch
    torch.cuda.synchronize()
    assert float(sink) == 0.0


@pytest.mark.parametrize("P,k", [(0, 1), (0, 40), (3, 61), (64, 64), (127, 1), (500, 289)])
def test_block_bf16_key_range_edges(hx, P, k):
    """No prior keys at all, one partial key tile, exact tile multiples, a one-key ragged tail."""
    _say(f"block bf16 P={P} k={k}")
    wl = _custom("bf16", B=2, grid=17, prev=13, P=P, C=128, heads=2)
    hb = hx.make_host_block(wl, 0, k=k)
    errs = hx.check_block(hb, hx.BF16_TOL)
    _say(f"   errors {errs}")


@pytest.mark.parametrize("dh_case", [(128, 2), (256, 2)])
@pytest.mark.parametrize("forced_split", [0, 3])
def test_block_bf16_peaked_attention_with_rising_scores(hx, dh_case, forced_split, monkeypatch):
    """Sharply peaked attention whose largest score keeps rising along the keys: the query projection is scaled
    up (scores spread over tens of nats) and the prior keys grow in length with their position, so that the
    softmax reference point of the kernel has to move several times while it walks the key tiles, also inside
    the runs of a split item."""
    C, heads = dh_case
    if forced_split:
        from paper_2602_01345_amd import Nova
        monkeypatch.setenv("NOVA_ATTN_SPLIT", str(forced_split))
        monkeypatch.setattr(hx, "_NOVA", Nova(0))
    _say(f"block bf16 peaked attention C={C} heads={heads} split={forced_split}")
    wl = _custom("bf16", B=2, grid=17, prev=13, P=1500, C=C, heads=heads)
    hb = hx.make_host_block(wl, 0, k=150)
    w = hb.weights["w_qkv"].to(torch.float32)
    w[:C] *= 24.0                                                     # query rows of [3C, C]
    hb.weights["w_qkv"] = w.to(hb.weights["w_qkv"].dtype)
    ramp = torch.linspace(0.25, 4.0, hb.k_prior.shape[1]).reshape(1, -1, 1)
    hb.k_prior = (hb.k_prior.to(torch.float32) * ramp).to(hb.k_prior.dtype)
    # the scores must really be spread: oracle-side check of the spread on one image and head
    x0 = hb.x[0].to(torch.float64)
    u = (x0 - x0.mean(-1, keepdim=True)) / torch.sqrt(x0.var(-1, unbiased=False, keepdim=True) + 1e-6)
    dh = C // heads
    q = (u @ hb.weights["w_qkv"].to(torch.float64)[:dh].T)            # head 0 queries, biases aside
    sc = (q @ hb.k_prior[0, :, :dh].to(torch.float64).T) / dh ** 0.5
    assert float(sc.max() - sc.median()) > 25.0, "the case no longer produces peaked attention"
    errs = hx.check_block(hb, hx.BF16_TOL)
    _say(f"   errors {errs}")


@pytest.mark.parametrize("split", [2, 3, 4])
def test_block_bf16_forced_key_splits(hx, split, monkeypatch):
    """The split-key attention path (partial sums merged by the combine kernel) with every split count."""
    from paper_2602_01345_amd import Nova
    monkeypatch.setenv("NOVA_ATTN_SPLIT", str(split))
    forced = Nova(0)                                   # the knob is read when a context is created
    monkeypatch.setattr(hx, "_NOVA", forced)
    wl = _custom("bf16", B=1, grid=20, prev=16, P=700, C=256, heads=2)      # 1100 keys = 18 tiles, dh = 128
    hb = hx.make_host_block(wl, 0, k=400)
    errs = hx.check_block(hb, hx.BF16_TOL)
    _say(f"   split {split}: errors {errs}")
    wl = _custom("bf16", B=2, grid=12, prev=8, P=260, C=128, heads=2)       # dh = 64, ragged last tile
    hb = hx.make_host_block(wl, 0, k=77)
    hx.check_block(hb, hx.BF16_TOL)


@pytest.mark.parametrize("knob,value", [("NOVA_ATTN_CFG", "2"), ("NOVA_ATTN_CFG", "3"), ("NOVA_ATTN_CFG", "4"),
                                        ("NOVA_GEMM_CFG", "0"), ("NOVA_GEMM_CFG", "1"), ("NOVA_GEMM_CFG", "2"),
                                        ("NOVA_GEMM_CFG", "5"), ("NOVA_GEMM_CFG", "6"), ("NOVA_GEMM_PARTS", "0"),
                                        ("NOVA_GEMM_PERSIST", "0")])
def test_block_bf16_with_every_tuning_knob(hx, knob, value, monkeypatch):
    """The kernel shapes that only an environment knob selects (other attention workgroup shapes, every GEMM tile
    configuration forced, no two-launch row plans, one workgroup per tile) compute the same block."""
    from paper_2602_01345_amd import Nova
    monkeypatch.setenv(knob, value)
    monkeypatch.setattr(hx, "_NOVA", Nova(0))          # the knobs are read when a context is created
    _say(f"block bf16 with {knob}={value}")
    for C, heads, P, k in ((128, 2, 300, 150), (512, 4, 700, 289)):      # dh = 64 and dh = 128, ragged everywhere
        wl = _custom("bf16", B=2, grid=17, prev=13, P=P, C=C, heads=heads)
        errs = hx.check_block(hx.make_host_block(wl, 0, k=k), hx.BF16_TOL)
        _say(f"   C={C}: errors {errs}")


@pytest.mark.parametrize("cfg", [None, "2", "6"])
def test_block_bf16_value_append_at_every_alignment(hx, cfg, monkeypatch):
    """The QKV projection's epilogue writes the value columns in 16-byte groups of eight cache slots: every offset of
    the first appended slot inside such a group, keep counts that leave partial groups at both ends, an image boundary
    inside a tile, and a feature count that puts query, key and value columns into one tile (C = 320 with 256- and
    128-column tiles).  The harness also checks that no slot outside the appended range is written."""
    from paper_2602_01345_amd import Nova
    if cfg is not None:
        monkeypatch.setenv("NOVA_GEMM_CFG", cfg)
        monkeypatch.setattr(hx, "_NOVA", Nova(0))
    _say(f"value append alignments, tile configuration {cfg}")
    for P, k in ((64, 40), (65, 290), (66, 7), (67, 300), (132, 129), (133, 8), (134, 261), (135, 1)):
        wl = _custom("bf16", B=2, grid=18, prev=12, P=P, C=320, heads=5)
        errs = hx.check_block(hx.make_host_block(wl, 0, k=k), hx.BF16_TOL)
        _say(f"   P={P} k={k}: errors {errs}")


@pytest.mark.parametrize("ksplit", ["0", "2", "4", None])
def test_block_bf16_ffn_down_projection_with_k_slices(hx, ksplit, monkeypatch):
    """The FFN down projection with large tiles and K = 4096 cut into 2 or 4 slices (fp32 partial sums, second
    pass), forced on, forced off, and as the launcher chooses (600 rows: slices; 1400 rows: none)."""
    from paper_2602_01345_amd import Nova
    if ksplit is not None:
        monkeypatch.setenv("NOVA_GEMM_KSPLIT", ksplit)
        monkeypatch.setattr(hx, "_NOVA", Nova(0))
    _say(f"block bf16 C=1024 F=4096, K slices of the down projection: {ksplit}")
    for k in (300, 700):
        wl = _custom("bf16", B=2, grid=28, prev=20, P=500, C=1024, heads=8)
        errs = hx.check_block(hx.make_host_block(wl, 0, k=k), hx.BF16_TOL)
        _say(f"   M={2 * k}: errors {errs}")


def test_step_with_look_ahead_selection_equals_the_sequential_step(hx):
    """run_step enqueues every block's entropy + selection one block ahead on a second stream; the outputs must
    be those of the plain sequence, bit for bit, also when the step is repeated."""
    wl = WL.Workload("steps", "bf16", B=2, C=128, heads=2, L=4, V=256, keep_hi=.7, keep_lo=.3,
                     scales=(WL.Scale(grid=12, prev_grid=9, kv_len=130),), seed=11)
    runner = None
    for j in range(wl.L):
        r, st, x = hx.to_gpu(hx.make_host_block(wl, j))
        if runner is None:
            runner = r
        else:
            runner.add_block(st)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for st in runner.blocks for t in (st.entropy, st.kept_idx, st.keep_mask, st.out, st.cache_new)]

    def poison():
        for st in runner.blocks:
            st.out.fill_(float("nan"))
            st.entropy.fill_(-1.0)
            st.kept_idx.fill_(-7)
            st.keep_mask.fill_(9)

    runner.run_step(x, overlap_selection=False)
    ref = snapshot()
    for rep in range(3):
        poison()
        runner.run_step(x, overlap_selection=True)
        got = snapshot()
        assert all(torch.equal(a, b) for a, b in zip(ref, got)), f"repeat {rep}"


def test_block_is_deterministic(hx):
    """Two runs on the same inputs give the same bits (no floating-point atomics anywhere on the path), the
    scale mean entropy included: it decides an integer keep count downstream."""
    wl = _custom("bf16", B=2, grid=24, prev=18, P=900, C=256, heads=4)
    hb = hx.make_host_block(wl, 0, k=300)
    outs = []
    for _ in range(2):
        runner, st, x = hx.to_gpu(hb)
        runner.run_block(st, x)
        mean = torch.empty(wl.B, dtype=torch.float32, device="cuda")
        H2 = torch.empty_like(st.entropy)
        hx.nova().entropy(st.logits, H2, mean)
        torch.cuda.synchronize()
        outs.append([t.clone() for t in (st.entropy, st.kept_idx, st.keep_mask, st.y_kept, st.out, st.cache_new,
                                         st.k_cache, st.v_cache, H2, mean)])
    for a, b in zip(*outs):
        assert torch.equal(a, b)
    assert torch.equal(outs[0][0], outs[0][8])


def test_mean_entropy_is_the_same_bits_on_every_run(hx):
    """cfg5-sized logits (2 x 4096 tokens): the mean is summed in a fixed order, so ten runs agree bit for bit,
    and it equals the float64 mean of the entropies the kernel wrote to fp32 rounding."""
    wl = WL.WORKLOADS["cfg5"]
    logits = WL.make_logits(wl, 3).cuda()
    H = torch.empty((wl.B, wl.last.N), dtype=torch.float32, device="cuda")
    means = []
    for _ in range(10):
        mean = torch.full((wl.B,), float("nan"), dtype=torch.float32, device="cuda")
        hx.nova().entropy(logits, H, mean)
        torch.cuda.synchronize()
        means.append(mean.cpu().numpy().copy())
    for m in means[1:]:
        assert np.array_equal(m, means[0])
    want = O.mean_entropy(H.cpu().numpy().astype(np.float64))
    assert np.allclose(means[0], want, rtol=2e-6, atol=0)


def test_tile_walking_gemm_workgroups_give_the_same_bits_as_one_workgroup_per_tile(hx, monkeypatch):
    """At the largest workload the projections with more tiles than CUs run one workgroup per CU that walks its
    tiles; every tile is still summed in the same order, so the block's outputs are the same bits as with one
    workgroup per tile (NOVA_GEMM_PERSIST=0)."""
    from paper_2602_01345_amd import Nova
    wl = WL.WORKLOADS["cfg5"]
    hb = hx.make_host_block(wl, 0)
    _say(f"cfg5 block 0, k={hb.k}: tile-walking workgroups against one workgroup per tile")
    outs = []
    for persist in ("1", "0"):
        monkeypatch.setenv("NOVA_GEMM_PERSIST", persist)
        monkeypatch.setattr(hx, "_NOVA", Nova(0))
        runner, st, x = hx.to_gpu(hb)
        runner.run_block(st, x)
        torch.cuda.synchronize()
        outs.append([t.clone() for t in (st.y_kept, st.out, st.cache_new)])
        del runner, st, x
    for a, b in zip(*outs):
        assert torch.equal(a, b)
