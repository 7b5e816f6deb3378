"""Chained multi-scale run (dense scales build the caches, pruned scales reuse them) against the
oracle applied step by step (Sec. 3.3: "Adaptive Acceleration Activation" decides where pruning
starts, "Residual Cache Reuse" chains the caches from scale to scale).

The oracle side keeps its own K/V rows and residual caches from scale to scale; between calls it
stores them in the workload's storage type (the tensors the method keeps are stored tensors), so
for bf16 both sides round at the same places.  Selection uses the entropies and keep counts the
device produced, as in the single-block tests."""
import numpy as np
import pytest
import torch

import harness as Hn
import workloads as WL
from oracle import nova_controller as K
from oracle import nova_oracle as O
from paper_2602_01345_amd import unpack_k_rows, unpack_v_rows
from paper_2602_01345_amd.image import ImageRunner


def _store(a: np.ndarray, dtype: torch.dtype) -> np.ndarray:
    """Round a float64 array to the storage type and back."""
    return torch.from_numpy(np.ascontiguousarray(a)).to(dtype).to(torch.float64).numpy()


def _workload(dtype, B, C, heads, L, V, grids):
    scales = tuple(WL.Scale(grid=g, prev_grid=grids[t - 1] if t else g, kv_len=sum(q * q for q in grids[:t]))
                   for t, g in enumerate(grids))
    return WL.Workload(f"chain-{dtype}", dtype, B=B, C=C, heads=heads, L=L, V=V, keep_hi=0.7, keep_lo=0.4,
                       scales=scales, seed=3)


def _run_chain(dtype, B, C, heads, L, V, grids, first_pruned, tol, controller, variants=False, interp="bilinear"):
    wl = _workload(dtype, B, C, heads, L, V, grids)
    tdt = WL.torch_dtype(dtype)
    weights_h = [WL.make_weights(wl, j) for j in range(L)]
    weights_d = [{n: t.cuda() for n, t in w.items()} for w in weights_h]
    W64 = [{n: Hn.f64(t) for n, t in w.items()} for w in weights_h]
    var_d, var_kw = None, [{} for _ in range(L)]
    if variants:
        # modulation + gates, unit-length q/k and tanh GELU in every block (the key cache then holds unit-length
        # keys from the first scale on, as both sides append them)
        from paper_2602_01345_amd import BlockVariant
        gen = [WL.make_block_variant(wl, j) for j in range(L)]
        var_d = [BlockVariant(gelu_tanh=True, qk_scale=g["qk_scale"].cuda(), ada=g["ada"].cuda()) for g in gen]
        var_kw = [dict(gelu_form="tanh", qk_scale=Hn.f64(g["qk_scale"]), ada=Hn.f64(g["ada"])) for g in gen]
    runner = ImageRunner(Hn.nova(), B=B, C=C, heads=heads, grids=grids, dtype=tdt, weights=weights_d,
                         variants=var_d, interp={"bilinear": 0, "nearest": 1, "bicubic": 2}[interp])

    # the oracle's own K/V rows, per block and per image (the images' cache lengths drift apart once they keep
    # different numbers of tokens)
    k_prior = [[np.zeros((0, C)) for _ in range(B)] for _ in range(L)]
    v_prior = [[np.zeros((0, C)) for _ in range(B)] for _ in range(L)]
    cache = [None] * L
    cache_grid = None
    worst = 0.0
    counts_seen = []

    def padded(rows):
        Pmax = max(a.shape[0] for a in rows)
        outp = np.zeros((B, Pmax, C))
        for b, a in enumerate(rows):
            outp[b, :a.shape[0]] = a
        return outp

    for t, g in enumerate(grids):
        s = wl.scales[t]
        N = g * g
        x_h = WL.make_x(wl, s)
        logits_h = [WL.make_logits(wl, j, s) for j in range(L)]
        pruned = t >= first_pruned
        kw = {}
        if pruned:
            if controller:
                # scale-linkage ratios of the images: scale t relative to t* = first_pruned (1-based t* + 1 = t + 1),
                # a different growth rate per image, so every image has its own ratio
                r = [K.scale_ratio(t + 1, first_pruned, 0.35 * (b + 1) - 0.5, 0.8, 0.1) for b in range(B)]
                kw["ratio_t"] = torch.tensor(r, dtype=torch.float32, device="cuda")
            else:
                kw["k_table"] = [WL.keep_count(wl.keep_ratio(j), N) for j in range(L)]
        res = runner.run_scale(t, x_h.cuda(), logits=[a.cuda() for a in logits_h], keep_cache=t >= first_pruned - 1,
                               inspect=True, **kw)
        torch.cuda.synchronize()

        x = Hn.f64(x_h)
        hbar_layers = []
        for j in range(L):
            if pruned and controller:
                k_rows = [int(v) for v in res.k[j].cpu().tolist()]          # every image's own count
            else:
                k_rows = [int(res.k[j])] * B
            kpitch = N if (pruned and controller) else k_rows[0]
            if pruned:
                H_gpu = res.block_entropy[j].cpu().numpy()
                assert Hn.entropy_ok(H_gpu, O.entropy(Hn.f64(logits_h[j])))
                if controller:
                    hbar_layers.append(H_gpu.astype(np.float64).mean(axis=1))
                    for b in range(B):
                        rt = float(kw["ratio_t"][b])
                        want = K.layer_ratio(rt, [h[b] for h in hbar_layers])
                        # the device evaluates the ratio in fp32 (|error| <= 1e-5 (1 + |ratio|)): its count is the
                        # exact rule's unless ratio * N comes that close to an integer
                        prod = K.clamp_ratio(want) * N
                        slack = 2e-5 * (1.0 + abs(want)) * N
                        near = abs(prod - round(prod)) <= slack
                        assert abs(k_rows[b] - K.keep_count(want, N)) <= (1 if near else 0), (t, j, b, k_rows, want)
                    counts_seen.append(tuple(k_rows))
                idx, mask = O.select(H_gpu, k_rows)
                full = np.full((B, kpitch), -1, dtype=np.int64)
                full[:, :idx.shape[1]] = idx
                idx = full
                assert np.array_equal(res.block_idx[j].cpu().numpy(), idx), (t, j)
            else:
                idx = np.tile(np.arange(N), (B, 1))
            P_rows = [a.shape[0] for a in k_prior[j]]
            y, kn, vn = O.pruned_block(x, idx, W64[j], padded(k_prior[j]), padded(v_prior[j]), heads, kv_rows=P_rows,
                                       **var_kw[j])
            if cache[j] is None:
                assert k_rows == [N] * B
                out, cn = O.merge_cache(x, y, idx, np.zeros((B, N, C)), g, g, g, g)
            else:
                out, cn = O.merge_cache(x, y, idx, cache[j], cache_grid, cache_grid, g, g, interp=interp)
            out, cn, kn, vn = (_store(a, tdt) for a in (out, cn, kn, vn))
            # compare what the device produced and stored
            errs = [Hn.nerr(res.block_out[j], out)]
            k_scale, v_scale = max(np.max(np.abs(kn)), 1e-30), max(np.max(np.abs(vn)), 1e-30)
            for b in range(B):
                P, k = P_rows[b], k_rows[b]
                if k:
                    gk = Hn.f64(unpack_k_rows(runner.k_cache[j], P, P + k)[b])
                    gv = Hn.f64(unpack_v_rows(runner.v_cache[j], P, P + k)[b])
                    errs += [float(np.max(np.abs(gk - kn[b, :k])) / k_scale), float(np.max(np.abs(gv - vn[b, :k])) / v_scale)]
                k_prior[j][b] = np.concatenate([k_prior[j][b], kn[b, :k]], axis=0)
                v_prior[j][b] = np.concatenate([v_prior[j][b], vn[b, :k]], axis=0)
            if res.block_cache[j] is not None:
                errs.append(Hn.nerr(res.block_cache[j], cn, scale_ref=out))
            worst = max(worst, *errs)
            assert max(errs) <= tol, (t, j, errs)
            if t >= first_pruned - 1:
                cache[j] = cn
            x = out
        if t >= first_pruned - 1:
            cache_grid = g
        # the device's own per-image cache lengths, and the host's upper bound
        for j in range(L):
            lens = [a.shape[0] for a in k_prior[j]]
            assert runner.kv_rows[j].cpu().tolist() == lens
            assert runner.kv_len[j] >= max(lens)
    if controller:
        # the images really did keep different numbers of tokens
        assert any(len(set(c)) == B for c in counts_seen), counts_seen
    return worst


@pytest.mark.gpu
@pytest.mark.parametrize("controller", [False, True])
def test_chain_f32(controller):
    # two dense scales, three pruned ones; fp32 throughout
    worst = _run_chain("f32", B=3, C=64, heads=2, L=2, V=128, grids=[2, 3, 4, 6, 8], first_pruned=2,
                       tol=Hn.F32_TOL * 4, controller=controller)
    assert worst > 0.0


@pytest.mark.gpu
@pytest.mark.parametrize("controller", [False, True])
def test_chain_bf16(controller):
    # matrix-core path: dh = 64, several key tiles and a ragged tail at every scale
    _run_chain("bf16", B=3, C=128, heads=2, L=3, V=256, grids=[3, 5, 8, 11, 13], first_pruned=2,
               tol=Hn.BF16_TOL * 1.5, controller=controller)


@pytest.mark.gpu
def test_controller_scale_runs_without_a_host_round_trip():
    """A pruned scale in controller mode (per-image counts from nova_layer_ratio through selection, block and
    merge) is recorded into a HIP graph: stream capture fails on anything that waits for the device, so a
    successful capture shows that no count visits the host.  One replay must give the bits of the eager run."""
    dtype, B, C, heads, L, V = "bf16", 3, 128, 2, 2, 256
    grids, first_pruned = [3, 5, 8, 11], 2
    wl = _workload(dtype, B, C, heads, L, V, grids)
    tdt = WL.torch_dtype(dtype)
    weights_d = [{n: t.cuda() for n, t in WL.make_weights(wl, j).items()} for j in range(L)]
    runners = [ImageRunner(Hn.nova(), B=B, C=C, heads=heads, grids=grids, dtype=tdt, weights=weights_d) for _ in range(2)]
    xs = [WL.make_x(wl, wl.scales[t]).cuda() for t in range(len(grids))]
    logits = [[WL.make_logits(wl, j, wl.scales[t]).cuda() for j in range(L)] for t in range(len(grids))]
    ratio = torch.tensor([0.25, 0.5, 0.75], dtype=torch.float32, device="cuda")
    for r in runners:
        for t in range(first_pruned):
            r.run_scale(t, xs[t], logits=logits[t], keep_cache=t >= first_pruned - 1)
    t = first_pruned
    # the eager run; its workspace is allocated here, outside any capture
    eager = runners[0].run_scale(t, xs[t], logits=logits[t], ratio_t=ratio)
    torch.cuda.synchronize()
    runners[1]._ensure_workspace(runners[1]._shape(grids[t] ** 2, 0, grids[t] ** 2))
    state = runners[1]._state.clone()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        captured = runners[1].run_scale(t, xs[t], logits=logits[t], ratio_t=ratio)
    runners[1]._state.copy_(state)
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(eager.out, captured.out)
    for a, b in zip(eager.block_cache, captured.block_cache):
        assert torch.equal(a, b)
    counts = [k.cpu().tolist() for k in captured.k]
    assert counts == [k.cpu().tolist() for k in eager.k]
    assert all(len(set(c)) == B for c in counts), counts
    for j in range(L):
        assert torch.equal(runners[0].kv_rows[j], runners[1].kv_rows[j])
        assert torch.equal(runners[0].k_cache[j], runners[1].k_cache[j])


@pytest.mark.gpu
@pytest.mark.parametrize("dtype,interp", [("f32", "bicubic"), ("bf16", "nearest"), ("bf16", "bicubic")])
def test_chain_with_block_variants_and_other_interpolation(dtype, interp):
    """The chained run with every block built the other way (modulation and gates, unit-length q/k, tanh GELU)
    and the residual cache interpolated with another kernel."""
    if dtype == "f32":
        _run_chain("f32", B=2, C=64, heads=2, L=2, V=128, grids=[2, 3, 4, 6, 8], first_pruned=2,
                   tol=Hn.F32_TOL * 4, controller=False, variants=True, interp=interp)
    else:
        _run_chain("bf16", B=2, C=128, heads=2, L=3, V=256, grids=[3, 5, 8, 11, 13], first_pruned=2,
                   tol=Hn.BF16_TOL * 1.5, controller=False, variants=True, interp=interp)


@pytest.mark.gpu
def test_planned_scales_replay_as_graphs():
    """Planned execution: the eager launches of every scale, then the same scales replayed as HIP
    graphs several times with unrelated eager work and synchronisations in between; every replay
    must reproduce the eager results bit for bit (the kernels on this path are deterministic)."""
    dtype, B, C, heads, L, V = "bf16", 2, 128, 2, 3, 256
    grids, first_pruned = [2, 4, 6, 9, 12], 3
    wl = _workload(dtype, B, C, heads, L, V, grids)
    tdt = WL.torch_dtype(dtype)
    weights_d = [{n: t.cuda() for n, t in WL.make_weights(wl, j).items()} for j in range(L)]
    runner = ImageRunner(Hn.nova(), B=B, C=C, heads=heads, grids=grids, dtype=tdt, weights=weights_d)
    logits = {t: [WL.make_logits(wl, j, wl.scales[t]).cuda() for j in range(L)] for t in range(first_pruned, len(grids))}
    tables = {t: [WL.keep_count(wl.keep_ratio(j), grids[t] ** 2) for j in range(L)] for t in range(first_pruned, len(grids))}
    plans = runner.plan_image(tables, logits, first_cache_scale=first_pruned - 1)
    for p in plans:
        p.x.copy_(WL.make_x(wl, wl.scales[p.t]).cuda())

    def snapshot():
        torch.cuda.synchronize()
        snap = []
        for p in plans:
            snap.append([o.clone() for o in p.out] + [c.clone() for c in p.cache_new if c is not None])
        snap.append([k.clone() for k in runner.k_cache] + [v.clone() for v in runner.v_cache])
        return snap

    for p in plans:                                   # eager image
        runner.enqueue(p)
    ref = snapshot()
    # the planned path must agree with the per-call path of the other tests
    other = ImageRunner(Hn.nova(), B=B, C=C, heads=heads, grids=grids, dtype=tdt, weights=weights_d)
    for p in plans:
        kw = {"k_table": tables[p.t], "logits": logits[p.t]} if p.t in tables else {}
        res = other.run_scale(p.t, p.x, keep_cache=p.t >= first_pruned - 1, **kw)
        assert torch.equal(res.out, p.out[-1]), p.t
    for p in plans:
        runner.capture(p)
    scratch = torch.randn(1 << 20, device="cuda")
    for rep in range(3):
        for p in plans:                               # poison the outputs so a replay that does nothing is seen
            for o in p.out:
                o.fill_(float("nan"))
        for k in runner.k_cache:
            k.zero_()
        for p in plans:
            runner.launch(p)
            scratch = scratch * 1.0001 + 1.0          # unrelated eager work between the replays
        other.run_scale(0, plans[0].x)                # eager library launches too
        got = snapshot()
        for a, b in zip(ref, got):
            for u, v in zip(a, b):
                assert torch.equal(u, v), f"replay {rep} differs from the eager run"
