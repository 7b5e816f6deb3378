"""Test-side glue: moves a seeded workload block to the GPU, runs the HIP path through the
C ABI, runs the oracle on the same bytes, and measures the differences."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np
import torch

import workloads as WL
from oracle import nova_oracle as O
from paper_2602_01345_amd import BlockVariant, Nova, pack_k_cache, pack_v_cache, unpack_k_rows, unpack_v_rows
from paper_2602_01345_amd.step import BlockState, StepRunner

ENTROPY_RTOL, ENTROPY_ATOL = 1e-5, 1e-7     # fp32 entropies: |dH| <= 1e-5 |H| + 1e-7
BF16_TOL = 2e-2                             # bf16 tensors: max|d| / max|ref|
F32_TOL = 2e-5                              # fp32 block tensors: max|d| / max|ref| (K <= 256 fp32 accumulations)

_NOVA = None


def nova() -> Nova:
    global _NOVA
    if _NOVA is None:
        _NOVA = Nova(0)
    return _NOVA


def f64(t) -> np.ndarray:
    if isinstance(t, torch.Tensor):
        return t.detach().cpu().to(torch.float64).numpy()
    return np.asarray(t, dtype=np.float64)


def nerr(got, ref, scale_ref=None) -> float:
    """max|got - ref| / max|scale_ref| (scale_ref defaults to ref)."""
    got, ref = f64(got), f64(ref)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), "non-finite values in the GPU result"
    denom = np.max(np.abs(ref if scale_ref is None else f64(scale_ref)))
    return float(np.max(np.abs(got - ref)) / (denom if denom > 0 else 1.0))


def entropy_ok(got, ref) -> bool:
    got, ref = f64(got), f64(ref)
    return bool(np.all(np.abs(got - ref) <= ENTROPY_RTOL * np.abs(ref) + ENTROPY_ATOL))


@dataclass
class HostBlock:
    wl: WL.Workload
    scale: WL.Scale
    k: int
    logits: torch.Tensor
    x: torch.Tensor
    weights: Dict[str, torch.Tensor]
    k_prior: torch.Tensor
    v_prior: torch.Tensor
    cache_prev: torch.Tensor
    # block variations: any of "gelu_tanh" (bool), "qk_scale" ([heads] fp32), "ada" ([B, 6, C]), "cross" (dict of
    # projections and the condition tokens' keys / values [B, Lt, C]); None = base block
    variant: Optional[Dict[str, object]] = None


def make_host_block(wl: WL.Workload, j: int, scale: Optional[WL.Scale] = None, k: Optional[int] = None,
                    variant: Optional[set] = None, text_len: int = 77) -> HostBlock:
    """`variant`: a subset of {"gelu_tanh", "qk_norm", "ada", "cross"} switching block variations on."""
    s = scale or wl.last
    kp, vp = WL.make_kv_prior(wl, j, s)
    var = None
    if variant:
        gen = WL.make_block_variant(wl, j, text_len)
        var = {}
        if "cross" in variant:
            var["cross"] = gen["cross"]
        if "gelu_tanh" in variant:
            var["gelu_tanh"] = True
        if "ada" in variant:
            var["ada"] = gen["ada"]
        if "qk_norm" in variant:
            var["qk_scale"] = gen["qk_scale"]
            # the cache of such a model holds unit-length keys: rescale the generated prior rows per head
            # (in float32, stored back in the workload's dtype; both sides then read the same stored rows)
            B, P, C = kp.shape
            kh = kp.to(torch.float32).reshape(B, P, wl.heads, C // wl.heads)
            kp = torch.nn.functional.normalize(kh, dim=-1).reshape(B, P, C).to(kp.dtype)
    return HostBlock(wl, s, wl.k(j, s) if k is None else k, WL.make_logits(wl, j, s), WL.make_x(wl, s),
                     WL.make_weights(wl, j), kp, vp, WL.make_cache_prev(wl, j, s), var)


def to_gpu(hb: HostBlock, poison: bool = False):
    """Uploads one block; with poison=True every cache row the call must not read is NaN."""
    wl, s = hb.wl, hb.scale
    dev = "cuda"
    cap = wl.kv_capacity(s)
    runner = StepRunner(nova(), B=wl.B, grid=s.grid, prev_grid=s.prev_grid, C=wl.C, heads=wl.heads,
                        kv_len=s.kv_len, kv_capacity=cap, dtype=WL.torch_dtype(wl.dtype), ffn_mult=wl.ffn_mult)
    fill = float("nan") if poison else 0.0
    st = BlockState(
        k=hb.k, logits=hb.logits.to(dev), weights={n: t.to(dev) for n, t in hb.weights.items()},
        k_cache=pack_k_cache(hb.k_prior.to(dev), wl.heads, cap, fill),
        v_cache=pack_v_cache(hb.v_prior.to(dev), wl.heads, cap, fill),
        cache_prev=hb.cache_prev.to(dev))
    if hb.variant is not None:
        qs, ada = hb.variant.get("qk_scale"), hb.variant.get("ada")
        cross = hb.variant.get("cross")
        if cross is not None:
            Lt = cross["k_text"].shape[1]
            cap_t = (Lt + 63) // 64 * 64
            cross = {"w_cq": cross["w_cq"].to(dev), "b_cq": cross["b_cq"].to(dev), "w_co": cross["w_co"].to(dev),
                     "b_co": cross["b_co"].to(dev), "text_len": Lt,
                     "k_text": pack_k_cache(cross["k_text"].to(dev), wl.heads, cap_t, fill),
                     "v_text": pack_v_cache(cross["v_text"].to(dev), wl.heads, cap_t, fill)}
        st.variant = BlockVariant(gelu_tanh=bool(hb.variant.get("gelu_tanh", False)),
                                  qk_scale=None if qs is None else qs.to(dev),
                                  ada=None if ada is None else ada.to(dev), cross=cross)
    runner.add_block(st)
    return runner, st, hb.x.to(dev)


def oracle_block(hb: HostBlock, H32: np.ndarray, rows=None):
    """Oracle results for the batch rows in `rows` (default all), selecting on the given fp32 entropies."""
    wl, s = hb.wl, hb.scale
    rows = list(range(wl.B)) if rows is None else list(rows)
    sel = lambda t: f64(t)[rows]
    idx, mask = O.select(np.asarray(H32)[rows], hb.k)
    W = {n: f64(t) for n, t in hb.weights.items()}
    x = sel(hb.x)
    kw = {}
    if hb.variant is not None:
        kw["gelu_form"] = "tanh" if hb.variant.get("gelu_tanh", False) else "erf"
        if hb.variant.get("qk_scale") is not None:
            kw["qk_scale"] = f64(hb.variant["qk_scale"])
        if hb.variant.get("ada") is not None:
            kw["ada"] = sel(hb.variant["ada"])
        if hb.variant.get("cross") is not None:
            c = hb.variant["cross"]
            kw["cross"] = {n: (sel(t) if n in ("k_text", "v_text") else f64(t)) for n, t in c.items()}
    y, kn, vn = O.pruned_block(x, idx[:, :hb.k], W, sel(hb.k_prior), sel(hb.v_prior), wl.heads, **kw)
    out, cn = O.merge_cache(x, y, idx[:, :hb.k], sel(hb.cache_prev), s.prev_grid, s.prev_grid, s.grid, s.grid)
    return dict(idx=idx, mask=mask, y=y, k_new=kn, v_new=vn, out=out, cache_new=cn)


def check_block(hb: HostBlock, tol: float, rows=None, poison: bool = True) -> Dict[str, float]:
    """Runs one block on the GPU and compares every output with the oracle; returns the errors."""
    wl, s = hb.wl, hb.scale
    runner, st, x = to_gpu(hb, poison=poison)
    runner.run_block(st, x)
    torch.cuda.synchronize()
    rows = list(range(wl.B)) if rows is None else list(rows)
    # entropy against the definition
    H_ref = O.entropy(f64(hb.logits)[rows])
    H_gpu = st.entropy.cpu().numpy()
    assert entropy_ok(H_gpu[rows], H_ref), "entropy outside 1e-5 rel + 1e-7 abs"
    # selection: same fp32 array on both sides, bit-exact
    ref = oracle_block(hb, H_gpu, rows)
    k = hb.k
    assert np.array_equal(st.keep_mask.cpu().numpy()[rows], ref["mask"]), "keep mask differs"
    if k > 0:
        assert np.array_equal(st.kept_idx.cpu().numpy()[rows, :k], ref["idx"][:, :k]), "kept index list differs"
    errs = {}
    P = s.kv_len
    if k > 0:
        errs["y_kept"] = nerr(st.y_kept[rows, :k], ref["y"])
        errs["k_new"] = nerr(unpack_k_rows(st.k_cache, P, P + k)[rows], ref["k_new"])
        errs["v_new"] = nerr(unpack_v_rows(st.v_cache, P, P + k)[rows], ref["v_new"])
    errs["out"] = nerr(st.out[rows], ref["out"])
    # cache_new = out - x is a difference of two stored tensors: its absolute error is that of
    # `out`, so it is measured on the scale of `out` (on kept rows the residual itself can be
    # far smaller than the bf16 spacing of the activations it is the difference of)
    errs["cache_new"] = nerr(st.cache_new[rows], ref["cache_new"], scale_ref=ref["out"])
    for name, e in errs.items():
        assert e <= tol, f"{name}: normalised max error {e:.3e} > {tol:.1e}"
    # the same absolute error on the residual's own scale (max|cache_new|), for the record: reported, and
    # bounded by the tolerance times the ratio of the two scales, which is the same statement as the line above
    errs["cache_new_own_scale"] = nerr(st.cache_new[rows], ref["cache_new"])
    # prior cache rows must be untouched
    assert torch.equal(unpack_k_rows(st.k_cache, 0, P).cpu(), hb.k_prior), "prior key rows were modified"
    assert torch.equal(unpack_v_rows(st.v_cache, 0, P).cpu(), hb.v_prior), "prior value rows were modified"
    if poison:
        # and so must every slot behind the appended rows (NaN poison, in both cache layouts)
        cap = wl.kv_capacity(s)
        assert bool(torch.isnan(unpack_k_rows(st.k_cache, P + k, cap)).all()), "key slots behind the appended rows were written"
        assert bool(torch.isnan(unpack_v_rows(st.v_cache, P + k, cap)).all()), "value slots behind the appended rows were written"
    return errs


def check_block_rows(hb: HostBlock, k_rows, kv_rows, tol: float, kpitch: Optional[int] = None) -> Dict[str, float]:
    """One block with per-image keep counts and per-image cache lengths on the device (nova_select with
    per-row counts -> nova_pruned_block_rows -> nova_merge_cache_rows) against the oracle's per-image form.
    Image b keeps k_rows[b] tokens and holds kv_rows[b] <= P prior rows; the row pitch defaults to N.  Cache rows
    the call must neither read nor write are NaN and must still be NaN afterwards."""
    wl, s = hb.wl, hb.scale
    B, N, C, P = wl.B, s.N, wl.C, s.kv_len
    kpitch = N if kpitch is None else kpitch
    assert len(k_rows) == B and len(kv_rows) == B and max(k_rows) <= kpitch and max(kv_rows) <= P
    dev = "cuda"
    n = nova()
    tdt = WL.torch_dtype(wl.dtype)
    cap = wl.kv_capacity(s)
    nan = float("nan")
    kc = pack_k_cache(hb.k_prior.to(dev), wl.heads, cap, nan)
    vc = pack_v_cache(hb.v_prior.to(dev), wl.heads, cap, nan)
    for b in range(B):                                   # rows past an image's own prior rows are not its cache
        kc[b, :, kv_rows[b]:] = nan
        vc[b, :, :, kv_rows[b]:] = nan
    kc0, vc0 = kc.clone(), vc.clone()
    x, logits = hb.x.to(dev), hb.logits.to(dev)
    W = {name: t.to(dev) for name, t in hb.weights.items()}
    H = torch.empty((B, N), dtype=torch.float32, device=dev)
    idx = torch.full((B, kpitch), -7, dtype=torch.int32, device=dev)
    mask = torch.full((B, N), 9, dtype=torch.uint8, device=dev)
    y = torch.full((B, kpitch, C), nan, dtype=tdt, device=dev)
    out = torch.full((B, N, C), nan, dtype=tdt, device=dev)
    cn = torch.full((B, N, C), nan, dtype=tdt, device=dev)
    kd = torch.tensor(k_rows, dtype=torch.int32, device=dev)
    kvd = torch.tensor(kv_rows, dtype=torch.int32, device=dev)
    kv_next = torch.full((B,), -1, dtype=torch.int32, device=dev)
    from paper_2602_01345_amd import BlockShape, NOVA_BF16, NOVA_F32
    shape = BlockShape(NOVA_BF16 if wl.dtype == "bf16" else NOVA_F32, B, N, C, wl.heads, P, cap, kpitch, wl.ffn_mult)
    ws = torch.empty(max(n.workspace_bytes(shape), 256), dtype=torch.uint8, device=dev)
    ws.view(torch.int16).fill_(0x7fc0)                   # NaN bit patterns (bf16; fp32 pairs too): stale workspace must not leak
    n.entropy(logits, H)
    n.select(H, kpitch, idx, mask, k_per_row=kd)
    n.pruned_block_rows(shape, W, None, kd, kvd, kv_next, x, idx, kc, vc, y, ws)
    n.merge_cache_rows(0, s.grid, s.grid, s.prev_grid, s.prev_grid, kpitch, kd, x, y, idx, mask,
                       hb.cache_prev.to(dev), out, cn)
    torch.cuda.synchronize()

    H_gpu = H.cpu().numpy()
    assert entropy_ok(H_gpu, O.entropy(f64(hb.logits)))
    ridx, rmask = O.select(H_gpu, list(k_rows))
    assert np.array_equal(mask.cpu().numpy(), rmask), "keep mask differs"
    kmax = ridx.shape[1]
    got_idx = idx.cpu().numpy()
    assert np.array_equal(got_idx[:, :kmax], ridx) and np.all(got_idx[:, kmax:] == -1), "kept index lists differ"
    assert kv_next.cpu().tolist() == [p + k for p, k in zip(kv_rows, k_rows)]
    full_idx = np.full((B, kpitch), -1, dtype=np.int64)
    full_idx[:, :kmax] = ridx
    Wd = {name: f64(t) for name, t in hb.weights.items()}
    ry, rk, rv = O.pruned_block(f64(hb.x), full_idx, Wd, f64(hb.k_prior), f64(hb.v_prior), wl.heads, kv_rows=kv_rows)
    rout, rcn = O.merge_cache(f64(hb.x), ry, full_idx, f64(hb.cache_prev), s.prev_grid, s.prev_grid, s.grid, s.grid)
    errs = {"out": nerr(out, rout), "cache_new": nerr(cn, rcn, scale_ref=rout)}
    y_scale = max(float(np.max(np.abs(ry))), 1e-30)
    k_scale = max(float(np.max(np.abs(rk))), 1e-30)
    v_scale = max(float(np.max(np.abs(rv))), 1e-30)
    ey = ek = ev = 0.0
    for b in range(B):
        k, Pb = k_rows[b], kv_rows[b]
        if k:
            ey = max(ey, float(np.max(np.abs(f64(y[b, :k]) - ry[b, :k]))) / y_scale)
            ek = max(ek, float(np.max(np.abs(f64(unpack_k_rows(kc, Pb, Pb + k)[b]) - rk[b, :k]))) / k_scale)
            ev = max(ev, float(np.max(np.abs(f64(unpack_v_rows(vc, Pb, Pb + k)[b]) - rv[b, :k]))) / v_scale)
        # everything outside [Pb, Pb + k) is bit for bit what it was (NaN poison included)
        for cache, before, dim in ((kc, kc0, 1), (vc, vc0, 2)):
            ibits = torch.int16 if cache.element_size() == 2 else torch.int32      # compare bit patterns (NaN poison)
            a, z = cache[b].view(ibits), before[b].view(ibits)
            sl_lo = [slice(None)] * 3
            sl_hi = [slice(None)] * 3
            sl_lo[dim], sl_hi[dim] = slice(0, Pb), slice(Pb + k, None)
            assert torch.equal(a[tuple(sl_lo)], z[tuple(sl_lo)]) and torch.equal(a[tuple(sl_hi)], z[tuple(sl_hi)]), \
                f"image {b}: cache rows outside its appended range were modified"
    errs.update(y_kept=ey, k_new=ek, v_new=ev)
    for name, e in errs.items():
        assert e <= tol, f"{name}: normalised max error {e:.3e} > {tol:.1e}"
    return errs
