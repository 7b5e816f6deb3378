"""GPU parity of the block variants behind nova_pruned_block_variant (per-image modulation and gates,
unit-length queries/keys with a per-head multiplier, tanh GELU, a cross-attention sub-layer: the ways the backbones of Sec. 4 build
their blocks) against the oracle's statement of the same variants, to the tolerances of the base block."""
import itertools

import numpy as np
import pytest
import torch

import workloads as WL

pytestmark = pytest.mark.gpu

ALL = ("gelu_tanh", "qk_norm", "ada", "cross")
SUBSETS = [set(c) for r in (1, 2, 4) for c in itertools.combinations(ALL, r)]


@pytest.fixture(scope="module")
def hx():
    import harness
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU and the built libnova.so (no fallback)")
    return harness


def _say(msg):
    print(msg, flush=True)


def _custom(dtype, B, grid, prev, P, C, heads, V=64, seed=9):
    return WL.Workload("custom", dtype, B=B, C=C, heads=heads, L=1, V=V, keep_hi=.5, keep_lo=.5,
                       scales=(WL.Scale(grid=grid, prev_grid=prev, kv_len=P),), seed=seed)


@pytest.mark.parametrize("variant", SUBSETS, ids=lambda v: "+".join(sorted(v)))
def test_variants_f32(hx, variant):
    _say(f"variant f32 {sorted(variant)}")
    wl = _custom("f32", B=3, grid=10, prev=7, P=45, C=48, heads=3)
    errs = hx.check_block(hx.make_host_block(wl, 0, k=37, variant=variant), hx.F32_TOL)
    _say(f"   errors {errs}")


@pytest.mark.parametrize("C,heads", [(128, 2), (256, 2)])
@pytest.mark.parametrize("variant", SUBSETS, ids=lambda v: "+".join(sorted(v)))
def test_variants_bf16(hx, variant, C, heads):
    # dh = 64 and 128; several row tiles with a ragged tail (k = 150), two key splits' worth of keys
    _say(f"variant bf16 C={C} heads={heads} {sorted(variant)}")
    wl = _custom("bf16", B=2, grid=17, prev=13, P=100, C=C, heads=heads)
    errs = hx.check_block(hx.make_host_block(wl, 0, k=150, variant=variant), hx.BF16_TOL)
    _say(f"   errors {errs}")


@pytest.mark.parametrize("k", [1, 289])
def test_variants_bf16_single_and_all_rows(hx, k):
    wl = _custom("bf16", B=2, grid=17, prev=13, P=0 if k == 289 else 64, C=128, heads=2)
    hx.check_block(hx.make_host_block(wl, 0, k=k, variant=set(ALL)), hx.BF16_TOL)


def test_variants_full_size_sampled_row(hx):
    """cfg5's last block (the launch configuration the benchmark times) with every variant on,
    one batch row checked against the oracle."""
    wl = WL.WORKLOADS["cfg5"]
    j = wl.L - 1
    _say(f"variant cfg5 block {j} k={wl.k(j)}")
    errs = hx.check_block(hx.make_host_block(wl, j, variant=set(ALL)), hx.BF16_TOL, rows=[1])
    _say(f"   errors {errs}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_no_variant_is_the_base_block_bit_for_bit(hx, dtype):
    from paper_2602_01345_amd import BlockVariant
    wl = _custom(dtype, B=2, grid=9, prev=6, P=64, C=128, heads=2)
    hb = hx.make_host_block(wl, 0, k=40)
    outs = []
    for var in (None, BlockVariant()):
        runner, st, x = hx.to_gpu(hb)
        st.variant = var
        runner.run_block(st, x)
        torch.cuda.synchronize()
        outs.append((st.y_kept.clone(), st.k_cache.clone(), st.v_cache.clone()))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_neutral_modulation_matches_the_base_block(hx):
    """shift = scale = 0 and gates = 1 go through the modulated kernels and must agree with the plain
    ones up to the rounding of the extra multiply-adds (bf16: identical; x * 1 + 0 is exact)."""
    from paper_2602_01345_amd import BlockVariant
    wl = _custom("bf16", B=2, grid=9, prev=6, P=64, C=128, heads=2)
    hb = hx.make_host_block(wl, 0, k=40)
    ada = torch.zeros(2, 6, 128, dtype=torch.bfloat16)
    ada[:, 2] = 1.0
    ada[:, 5] = 1.0
    outs = []
    for var in (None, BlockVariant(ada=ada.cuda())):
        runner, st, x = hx.to_gpu(hb)
        st.variant = var
        runner.run_block(st, x)
        torch.cuda.synchronize()
        outs.append(st.y_kept.clone())
    assert torch.equal(outs[0], outs[1])


def test_variant_argument_errors(hx):
    from paper_2602_01345_amd import BlockVariant, NovaError
    from paper_2602_01345_amd.binding import _Variant
    wl = _custom("bf16", B=2, grid=9, prev=6, P=64, C=128, heads=2)
    hb = hx.make_host_block(wl, 0, k=40, variant=set(ALL))
    runner, st, x = hx.to_gpu(hb)
    before = st.y_kept.fill_(7.0).clone()

    class Raw(BlockVariant):
        def __init__(self, raw):
            self.raw = raw

        def c_struct(self):
            return self.raw

    good = st.variant.c_struct()
    bad = [
        _Variant(2, 0, None, None),                                   # a flag that is neither 0 nor 1
        _Variant(0, 3, good.qk_scale, None),
        _Variant(0, 1, None, None),                                   # unit-length q/k without the multipliers
        _Variant(0, 0, None, good.ada + 2),                           # misaligned conditioning vectors
    ]
    for raw in bad:
        st.variant = Raw(raw)
        with pytest.raises(NovaError) as e:
            runner.run_block(st, x)
        assert e.value.code == -1
    torch.cuda.synchronize()
    assert torch.equal(st.y_kept, before), "a rejected call must leave the outputs untouched"


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("variant", [{"gelu_tanh"}, {"qk_norm"}, {"ada"}, {"cross"}], ids=lambda v: "+".join(sorted(v)))
def test_each_variant_moves_the_output_far_beyond_the_tolerance(hx, dtype, variant):
    """With the benchmark's small weights (std 0.02) both branches are small next to the residual stream, and
    a variant that the device ignored could hide inside the bf16 tolerance.  Here the weights are 8x larger
    (an exact scaling in bf16), so that the oracle's output with the variant differs from its output
    without it by many tolerances, and the device must follow the variant to pass."""
    from oracle import nova_oracle as O
    wl = _custom(dtype, B=2, grid=12, prev=9, P=70, C=128, heads=2)
    hb = hx.make_host_block(wl, 0, k=90, variant=variant)
    hb.weights = {n: (t * 8.0 if n.startswith("w_") else t) for n, t in hb.weights.items()}
    if "cross" in variant:
        hb.variant["cross"] = {n: (t * 8.0 if n.startswith("w_") else t) for n, t in hb.variant["cross"].items()}
    if "gelu_tanh" in variant:
        # the two GELU forms differ by at most 5e-4 in absolute terms: only fp32 can tell them apart
        if dtype == "bf16":
            pytest.skip("the GELU forms differ by less than the bf16 rounding of the hidden activations")
    tol = hx.BF16_TOL if dtype == "bf16" else hx.F32_TOL
    errs = hx.check_block(hb, tol)
    _say(f"   {dtype} {sorted(variant)} errors {errs}")
    # the oracle's own sensitivity to the variant on these inputs
    import numpy as np
    H = O.entropy(hx.f64(hb.logits)).astype(np.float32)
    with_var = hx.oracle_block(hb, H)["y"]
    hb.variant = None
    without = hx.oracle_block(hb, H)["y"]
    moved = hx.nerr(without, with_var)
    _say(f"   oracle moves by {moved:.3e} (tolerance {tol:.1e})")
    # the device is many times closer to the oracle with the variant than the oracle without it is
    assert moved > 4 * tol and moved > 20 * errs["y_kept"]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("text_len", [1, 64, 65, 300])
def test_cross_attention_condition_lengths(hx, dtype, text_len):
    """One condition token (softmax over a single key), a full tile, a tile plus one, several tiles."""
    C, heads = (48, 3) if dtype == "f32" else (128, 2)
    wl = _custom(dtype, B=2, grid=10, prev=7, P=45, C=C, heads=heads)
    hb = hx.make_host_block(wl, 0, k=37, variant={"cross"}, text_len=text_len)
    hx.check_block(hb, hx.BF16_TOL if dtype == "bf16" else hx.F32_TOL)


def test_cross_attention_argument_errors(hx):
    from paper_2602_01345_amd import BlockVariant, NovaError
    wl = _custom("bf16", B=2, grid=9, prev=6, P=64, C=128, heads=2)
    hb = hx.make_host_block(wl, 0, k=40, variant={"cross"})
    runner, st, x = hx.to_gpu(hb)
    good = st.variant

    class Raw(BlockVariant):
        def __init__(self, edit):
            self.edit = edit

        def c_struct(self):
            v = good.c_struct()
            self.edit(v)
            return v

    def drop(field):
        return lambda v: setattr(v, field, None)

    cases = [("no output projection", drop("w_co"), -1), ("no keys", drop("k_text"), -1), ("no values", drop("v_text"), -1),
             ("zero tokens", lambda v: setattr(v, "text_len", 0), -1),
             ("more tokens than capacity", lambda v: setattr(v, "text_len", 129), -1),
             ("misaligned keys", lambda v: setattr(v, "k_text", v.k_text + 2), -1),
             ("capacity not a multiple of the key tile", lambda v: setattr(v, "text_capacity", 100), -2)]
    before = st.y_kept.fill_(3.0).clone()
    for name, edit, code in cases:
        st.variant = Raw(edit)
        with pytest.raises(NovaError) as e:
            runner.run_block(st, x)
        assert e.value.code == code, name
    torch.cuda.synchronize()
    assert torch.equal(st.y_kept, before)
