"""Per-image keep counts on the device (Sec. 3.3, "Dual-Linkage Acceleration": the scale- and layer-linkage ratios are
per instance): nova_select with per-row counts -> nova_pruned_block_rows -> nova_merge_cache_rows against the oracle's
per-image form, and the chained controller run in which no count ever visits the host."""
import numpy as np
import pytest
import torch

import harness as Hn
import workloads as WL

pytestmark = pytest.mark.gpu


def _wl(dtype, B, grid, prev, P, C, heads, seed=9):
    return WL.Workload("rows", dtype, B=B, C=C, heads=heads, L=1, V=64, keep_hi=.5, keep_lo=.5,
                       scales=(WL.Scale(grid=grid, prev_grid=prev, kv_len=P),), seed=seed)


@pytest.mark.parametrize("C,heads", [(128, 2), (256, 2)])                       # dh = 64 and dh = 128
@pytest.mark.parametrize("k_rows,kv_rows", [([150, 0, 289], [100, 37, 64]), ([1, 37, 200], [0, 100, 1]),
                                            ([289, 289, 289], [100, 100, 100])])
def test_block_bf16_per_image_counts(C, heads, k_rows, kv_rows):
    print(f"per-image counts bf16 C={C} heads={heads} k={k_rows} kv={kv_rows}", flush=True)
    hb = Hn.make_host_block(_wl("bf16", 3, 17, 13, 100, C, heads), 0)
    errs = Hn.check_block_rows(hb, k_rows, kv_rows, Hn.BF16_TOL)
    print(f"   errors {errs}", flush=True)


@pytest.mark.parametrize("k_rows,kv_rows", [([37, 0, 100], [45, 3, 20]), ([100, 1, 0], [0, 45, 45])])
def test_block_f32_per_image_counts(k_rows, kv_rows):
    print(f"per-image counts f32 k={k_rows} kv={kv_rows}", flush=True)
    hb = Hn.make_host_block(_wl("f32", 3, 10, 7, 45, 48, 3), 0)
    errs = Hn.check_block_rows(hb, k_rows, kv_rows, Hn.F32_TOL)
    print(f"   errors {errs}", flush=True)


def test_block_bf16_per_image_counts_with_a_smaller_row_pitch():
    """The row pitch only has to cover the largest count."""
    hb = Hn.make_host_block(_wl("bf16", 3, 17, 13, 100, 128, 2), 0)
    Hn.check_block_rows(hb, [150, 3, 77], [100, 99, 0], Hn.BF16_TOL, kpitch=160)


def test_block_bf16_per_image_counts_large_tiles_with_dead_tiles():
    """2 x 1024 row slots through the large GEMM tiles: image 0 fills 600 of its slots, image 1 only 130, so whole
    256-row tiles hold no live row and are skipped; the attention's query blocks likewise."""
    hb = Hn.make_host_block(_wl("bf16", 2, 32, 24, 700, 512, 4), 0)
    errs = Hn.check_block_rows(hb, [600, 130], [700, 300], Hn.BF16_TOL)
    print(f"   errors {errs}", flush=True)


@pytest.mark.parametrize("split", [3, 4])
def test_block_bf16_per_image_counts_with_cut_attention_items(split, monkeypatch):
    """Cut attention items with per-image key counts: an image with few keys leaves some key runs empty (their
    partial results are all-zero with weight 0), an image without live queries leaves whole items to the merge pass."""
    from paper_2602_01345_amd import Nova
    monkeypatch.setenv("NOVA_ATTN_SPLIT", str(split))
    monkeypatch.setattr(Hn, "_NOVA", Nova(0))
    for C, heads in ((256, 2), (128, 2)):
        hb = Hn.make_host_block(_wl("bf16", 3, 20, 16, 700, C, heads), 0)
        errs = Hn.check_block_rows(hb, [400, 1, 0], [700, 0, 650], Hn.BF16_TOL)
        print(f"   split {split} C={C}: errors {errs}", flush=True)


def test_rows_entry_points_with_null_counts_are_the_uniform_calls():
    """nova_pruned_block_rows / nova_merge_cache_rows with NULL count arrays give the bits of the uniform calls."""
    hb = Hn.make_host_block(_wl("bf16", 2, 17, 13, 100, 128, 2), 0, k=150)
    runner, st, x = Hn.to_gpu(hb, poison=False)
    runner.run_block(st, x)
    torch.cuda.synchronize()
    ref = [t.clone() for t in (st.y_kept, st.out, st.cache_new, st.k_cache, st.v_cache)]
    runner2, st2, x2 = Hn.to_gpu(hb, poison=False)
    n = Hn.nova()
    n.entropy(st2.logits, st2.entropy)
    n.select(st2.entropy, st2.k, st2.kept_idx, st2.keep_mask)
    n.pruned_block_rows(runner2.shape(st2.k), st2.weights, None, None, None, None, x2, st2.kept_idx, st2.k_cache,
                        st2.v_cache, st2.y_kept, runner2._workspace)
    s = hb.scale
    n.merge_cache_rows(0, s.grid, s.grid, s.prev_grid, s.prev_grid, st2.k, None, x2, st2.y_kept, st2.kept_idx,
                       st2.keep_mask, st2.cache_prev, st2.out, st2.cache_new)
    torch.cuda.synchronize()
    for a, b in zip(ref, (st2.y_kept, st2.out, st2.cache_new, st2.k_cache, st2.v_cache)):
        assert torch.equal(a, b)


def test_rows_argument_errors():
    n = Hn.nova()
    from paper_2602_01345_amd import NovaError
    x = torch.zeros((1, 16, 128), dtype=torch.bfloat16, device="cuda")
    mask = torch.zeros((1, 16), dtype=torch.uint8, device="cuda")
    idx = torch.zeros((1, 16), dtype=torch.int32, device="cuda")
    kd = torch.zeros(1, dtype=torch.int32, device="cuda")
    out = torch.zeros_like(x)
    with pytest.raises(NovaError):        # per-image counts need the prior cache even at full pitch
        n.merge_cache_rows(0, 4, 4, 3, 3, 16, kd, x, x.clone(), idx, mask, None, out, None)
