"""Pins for the oracle's pruned block and residual-cache merge (CPU only).

The paper leaves Layer_j opaque (Sec. 3.3, Residual Cache Reuse, first
equation), so the block is pinned to what its stated structure fixes: keeping
every token equals an independently written dense block, per-token results do
not depend on the order of the kept list, degenerate weights give closed forms,
and each step agrees with a float64 library routine.  The merge is pinned to
the cache equations (same paragraph, second and third equations) and to closed
forms of half-pixel bilinear interpolation.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import nova_oracle as O


def _rand_block(rng, B=2, N=7, C=8, heads=2, P=3, Fm=4, bias=True):
    x = rng.standard_normal((B, N, C))
    W = {
        "w_qkv": rng.standard_normal((3 * C, C)) * 0.3, "b_qkv": rng.standard_normal(3 * C) * 0.1,
        "w_o": rng.standard_normal((C, C)) * 0.3, "b_o": rng.standard_normal(C) * 0.1,
        "w_fc1": rng.standard_normal((Fm * C, C)) * 0.3, "b_fc1": rng.standard_normal(Fm * C) * 0.1,
        "w_fc2": rng.standard_normal((C, Fm * C)) * 0.3, "b_fc2": rng.standard_normal(C) * 0.1,
    }
    if not bias:
        for n in ("b_qkv", "b_o", "b_fc1", "b_fc2"):
            W[n] = None
    kp = rng.standard_normal((B, P, C))
    vp = rng.standard_normal((B, P, C))
    return x, W, kp, vp


# ---- an independent dense block, scalar python loops, token by token --------
def _ln_scalar(v):
    n = len(v)
    mu = sum(v) / n
    var = sum((a - mu) ** 2 for a in v) / n
    return [(a - mu) / math.sqrt(var + 1e-6) for a in v]


def _linear_scalar(v, W, b):
    return [sum(W[o][i] * v[i] for i in range(len(v))) + (0.0 if b is None else b[o]) for o in range(len(W))]


def _dense_block_scalar(x, W, kp, vp, heads):
    """All N tokens of one batch row attend to P prior rows plus all N current rows."""
    N, C = len(x), len(x[0])
    dh = C // heads
    qkv = [_linear_scalar(_ln_scalar(x[i]), W["w_qkv"], W["b_qkv"]) for i in range(N)]
    keys = [list(r) for r in kp] + [r[C:2 * C] for r in qkv]
    vals = [list(r) for r in vp] + [r[2 * C:] for r in qkv]
    out = []
    for i in range(N):
        a = [0.0] * C
        for h in range(heads):
            q = qkv[i][h * dh:(h + 1) * dh]
            s = [sum(q[d] * kr[h * dh + d] for d in range(dh)) / math.sqrt(dh) for kr in keys]
            m = max(s)
            e = [math.exp(v - m) for v in s]
            Z = sum(e)
            for d in range(dh):
                a[h * dh + d] = sum(e[j] / Z * vals[j][h * dh + d] for j in range(len(keys)))
        o = _linear_scalar(a, W["w_o"], W["b_o"])
        x1 = [x[i][c] + o[c] for c in range(C)]
        hid = _linear_scalar(_ln_scalar(x1), W["w_fc1"], W["b_fc1"])
        hid = [0.5 * t * (1.0 + math.erf(t / math.sqrt(2.0))) for t in hid]
        f = _linear_scalar(hid, W["w_fc2"], W["b_fc2"])
        out.append([x1[c] + f[c] for c in range(C)])
    return out, [r[C:2 * C] for r in qkv], [r[2 * C:] for r in qkv]


@pytest.mark.parametrize("bias", [True, False])
def test_keep_all_equals_dense_block(bias):
    rng = np.random.default_rng(0)
    x, W, kp, vp = _rand_block(rng, bias=bias)
    B, N, C = x.shape
    idx = np.tile(np.arange(N), (B, 1))
    y, kn, vn = O.pruned_block(x, idx, W, kp, vp, heads=2)
    Wl = {n: (None if a is None else a.tolist()) for n, a in W.items()}
    for b in range(B):
        ref, rk, rv = _dense_block_scalar(x[b].tolist(), Wl, kp[b].tolist(), vp[b].tolist(), 2)
        np.testing.assert_allclose(y[b], np.array(ref), rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(kn[b], np.array(rk), rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(vn[b], np.array(rv), rtol=1e-10, atol=1e-12)


def test_pruned_block_matches_scalar_block_on_the_subset():
    """Kept tokens see only prior rows + kept rows: equal to the dense scalar
    block run on the gathered sub-sequence."""
    rng = np.random.default_rng(1)
    x, W, kp, vp = _rand_block(rng, B=1, N=9)
    idx = np.array([[1, 4, 5, 8]])
    y, _, _ = O.pruned_block(x, idx, W, kp, vp, heads=2)
    Wl = {n: a.tolist() for n, a in W.items()}
    ref, _, _ = _dense_block_scalar(x[0, idx[0]].tolist(), Wl, kp[0].tolist(), vp[0].tolist(), 2)
    np.testing.assert_allclose(y[0], np.array(ref), rtol=1e-10, atol=1e-12)


def test_kept_order_does_not_change_per_token_outputs():
    rng = np.random.default_rng(2)
    x, W, kp, vp = _rand_block(rng, B=1, N=10)
    idx = np.array([[0, 3, 4, 7, 9]])
    perm = np.array([3, 0, 4, 2, 1])
    y0, k0, v0 = O.pruned_block(x, idx, W, kp, vp, heads=2)
    y1, k1, v1 = O.pruned_block(x, idx[:, perm], W, kp, vp, heads=2)
    np.testing.assert_allclose(y1, y0[:, perm], rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(k1, k0[:, perm], rtol=1e-12)
    np.testing.assert_allclose(v1, v0[:, perm], rtol=1e-12)


def test_library_second_opinion_torch_float64():
    rng = np.random.default_rng(3)
    x, W, kp, vp = _rand_block(rng, B=2, N=12, C=16, heads=4, P=5)
    idx = np.array([[0, 2, 3, 7, 10, 11], [1, 2, 4, 5, 6, 9]])
    y, kn, vn = O.pruned_block(x, idx, W, kp, vp, heads=4)
    t = {n: torch.from_numpy(a) for n, a in W.items()}
    for b in range(2):
        xs = torch.from_numpy(x[b, idx[b]])
        u = F.layer_norm(xs, (16,), eps=1e-6)
        qkv = F.linear(u, t["w_qkv"], t["b_qkv"])
        q, kk, vv = qkv.split(16, dim=-1)
        K = torch.cat([torch.from_numpy(kp[b]), kk])
        V = torch.cat([torch.from_numpy(vp[b]), vv])
        hd = lambda a: a.reshape(a.shape[0], 4, 4).transpose(0, 1)      # [heads, rows, dh]
        a = F.scaled_dot_product_attention(hd(q), hd(K), hd(V)).transpose(0, 1).reshape(-1, 16)
        x1 = xs + F.linear(a, t["w_o"], t["b_o"])
        ref = x1 + F.linear(F.gelu(F.linear(F.layer_norm(x1, (16,), eps=1e-6), t["w_fc1"], t["b_fc1"])),
                            t["w_fc2"], t["b_fc2"])
        np.testing.assert_allclose(y[b], ref.numpy(), rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(kn[b], kk.numpy(), rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(vn[b], vv.numpy(), rtol=1e-10, atol=1e-12)


def test_degenerate_weights():
    rng = np.random.default_rng(4)
    x, W, kp, vp = _rand_block(rng, B=1, N=6, P=4)
    idx = np.array([[0, 2, 5]])
    C = x.shape[-1]
    # all-zero weights and biases: y = x on the kept rows
    Z = {n: np.zeros_like(a) for n, a in W.items()}
    y, _, _ = O.pruned_block(x, idx, Z, kp, vp, heads=2)
    np.testing.assert_allclose(y[0], x[0, idx[0]], atol=0)
    # zero query projection -> uniform attention -> mean of all value rows;
    # zero FFN1 weight -> FFN output = GELU(b1) W2^T + b2
    W2 = dict(W)
    W2["w_qkv"] = W["w_qkv"].copy(); W2["w_qkv"][:C] = 0
    W2["b_qkv"] = W["b_qkv"].copy(); W2["b_qkv"][:C] = 0
    W2["w_fc1"] = np.zeros_like(W["w_fc1"])
    y, kn, vn = O.pruned_block(x, idx, W2, kp, vp, heads=2)
    vmean = np.concatenate([vp[0], vn[0]]).mean(axis=0)
    x1 = x[0, idx[0]] + vmean @ W["w_o"].T + W["b_o"]
    g = np.array([0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in W["b_fc1"]])
    ref = x1 + g @ W["w_fc2"].T + W["b_fc2"]
    np.testing.assert_allclose(y[0], ref, rtol=1e-11, atol=1e-13)
    # constant value cache and zero value projection: attention output is that row
    W3 = dict(W)
    W3["w_qkv"] = W["w_qkv"].copy(); W3["w_qkv"][2 * C:] = 0
    W3["b_qkv"] = W["b_qkv"].copy(); W3["b_qkv"][2 * C:] = 0
    row = rng.standard_normal(C)
    vconst = np.tile(row, (1, 4, 1))
    W3["w_fc1"] = np.zeros_like(W["w_fc1"]); W3["b_fc1"] = np.zeros_like(W["b_fc1"])
    W3["b_fc2"] = np.zeros_like(W["b_fc2"])
    # the appended value rows are 0 and the P prior rows all equal `row`
    y, _, vn = O.pruned_block(x, idx, W3, kp, vconst, heads=2)
    assert np.all(vn == 0)
    a = (y[0] - x[0, idx[0]] - W["b_o"]) @ np.linalg.inv(W["w_o"].T)     # recover attention output
    # each head's output is t * row (0 < t < 1): a convex mix of `row` and the zero rows
    for h in range(2):
        sl = slice(h * 4, (h + 1) * 4)
        t = a[:, sl] / row[sl]
        assert np.allclose(t, t[:, :1], rtol=1e-8)
        assert np.all(t > 0) and np.all(t < 1)


def test_layer_norm_and_gelu_special_values():
    assert np.allclose(O.layer_norm(np.full((2, 5), 3.7)), 0.0)
    v = np.array([[1.0, 2.0, 3.0, 4.0]])
    ln = O.layer_norm(v)
    assert abs(ln.mean()) < 1e-15 and ln.var() == pytest.approx(1.25 / (1.25 + 1e-6), rel=1e-12)
    assert O.gelu(np.array([0.0]))[0] == 0.0
    assert O.gelu(np.array([1.0]))[0] == pytest.approx(0.8413447460685429, rel=1e-14)   # Phi(1)
    assert O.gelu(np.array([-1.0]))[0] == pytest.approx(-0.15865525393145707, rel=1e-13)


# ----------------------------------------------------------------------------
# residual cache reuse
# ----------------------------------------------------------------------------
def test_upsample_identity_constant_and_1x1():
    rng = np.random.default_rng(5)
    c = rng.standard_normal((2, 12, 3))
    np.testing.assert_allclose(O.bilinear_upsample(c, 3, 4, 3, 4), c, atol=1e-15)
    const = np.full((1, 6, 2), 2.5)
    np.testing.assert_allclose(O.bilinear_upsample(const, 2, 3, 5, 7), 2.5, atol=1e-15)
    one = rng.standard_normal((1, 1, 4))
    up = O.bilinear_upsample(one, 1, 1, 3, 3)
    np.testing.assert_allclose(up, np.tile(one, (1, 9, 1)), atol=0)


def test_upsample_1d_closed_form_2_to_4():
    a, b = 1.0, 5.0
    row = np.array([a, b]).reshape(1, 2, 1)
    up = O.bilinear_upsample(row, 1, 2, 1, 4).ravel()
    np.testing.assert_allclose(up, [a, 0.75 * a + 0.25 * b, 0.25 * a + 0.75 * b, b], rtol=1e-15)
    col = O.bilinear_upsample(row, 2, 1, 4, 1).ravel()
    np.testing.assert_allclose(col, up, rtol=1e-15)


def test_upsample_linear_ramp_interior_and_transpose_symmetry():
    hp, wp, h, w = 13, 13, 16, 16
    yy, xx = np.meshgrid(np.arange(hp), np.arange(wp), indexing="ij")
    ramp = (2.0 * yy - 3.0 * xx + 1.0).reshape(1, hp * wp, 1)
    up = O.bilinear_upsample(ramp, hp, wp, h, w).reshape(h, w)
    sy = (np.arange(h) + 0.5) * hp / h - 0.5
    sx = (np.arange(w) + 0.5) * wp / w - 0.5
    inside_y = (sy >= 0) & (sy <= hp - 1)
    inside_x = (sx >= 0) & (sx <= wp - 1)
    ref = 2.0 * sy[:, None] - 3.0 * sx[None, :] + 1.0
    sel = np.ix_(inside_y, inside_x)
    np.testing.assert_allclose(up[sel], ref[sel], rtol=1e-12, atol=1e-12)
    # interpolating the transposed field gives the transposed result (rows/columns are treated alike)
    rng = np.random.default_rng(6)
    c = rng.standard_normal((hp, wp))
    a = O.bilinear_upsample(c.reshape(1, -1, 1), hp, wp, h, w).reshape(h, w)
    bt = O.bilinear_upsample(c.T.reshape(1, -1, 1), wp, hp, w, h).reshape(w, h)
    np.testing.assert_allclose(a, bt.T, rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("hp,wp,h,w", [(13, 13, 16, 16), (3, 5, 7, 6), (48, 48, 64, 64), (5, 5, 4, 4)])
def test_upsample_library_second_opinion(hp, wp, h, w):
    rng = np.random.default_rng(7)
    c = rng.standard_normal((2, hp * wp, 3))
    up = O.bilinear_upsample(c, hp, wp, h, w)
    t = torch.from_numpy(c).reshape(2, hp, wp, 3).permute(0, 3, 1, 2)
    ref = F.interpolate(t, size=(h, w), mode="bilinear", align_corners=False, antialias=False)
    np.testing.assert_allclose(up, ref.permute(0, 2, 3, 1).reshape(2, h * w, 3).numpy(), rtol=1e-12, atol=1e-13)


def test_merge_rules():
    rng = np.random.default_rng(8)
    B, hp, wp, h, w, C = 2, 3, 3, 4, 4, 5
    N = h * w
    x = rng.standard_normal((B, N, C))
    cache_prev = rng.standard_normal((B, hp * wp, C))
    idx = np.array([[0, 5, 6, 15], [2, 3, 9, 10]])
    y = rng.standard_normal((B, 4, C))
    out, cn = O.merge_cache(x, y, idx, cache_prev, hp, wp, h, w)
    up = O.bilinear_upsample(cache_prev, hp, wp, h, w)
    for b in range(B):
        kept = set(idx[b].tolist())
        for i in range(N):
            if i in kept:
                s = idx[b].tolist().index(i)
                assert np.array_equal(out[b, i], y[b, s])              # kept rows: the block's output, copied
                np.testing.assert_allclose(cn[b, i], y[b, s] - x[b, i], atol=1e-15)
            else:
                np.testing.assert_allclose(out[b, i], x[b, i] + up[b, i], atol=1e-15)
                np.testing.assert_allclose(cn[b, i], up[b, i], atol=1e-15)
    np.testing.assert_allclose(cn, out - x, atol=0)
    # nothing kept: out = x + upsampled cache everywhere
    out0, cn0 = O.merge_cache(x, np.zeros((B, 0, C)), np.zeros((B, 0), dtype=np.int64), cache_prev, hp, wp, h, w)
    np.testing.assert_allclose(out0, x + up, atol=0)
    # everything kept: the prior cache is never read (NaN must not leak, None allowed)
    allidx = np.tile(np.arange(N), (B, 1))
    yall = rng.standard_normal((B, N, C))
    outN, cnN = O.merge_cache(x, yall, allidx, np.full_like(cache_prev, np.nan), hp, wp, h, w)
    assert np.array_equal(outN, yall) and not np.isnan(cnN).any()
    outN2, _ = O.merge_cache(x, yall, allidx, None, hp, wp, h, w)
    assert np.array_equal(outN2, yall)


# ---- block variants (conditioning by per-image vectors, unit-length q/k, tanh GELU) ---------
def _rand_variant(rng, B, C, heads):
    ada = rng.standard_normal((B, 6, C)) * 0.3
    ada[:, 2] += 1.0
    ada[:, 5] += 1.0                                   # gates around 1
    qk_scale = rng.uniform(2.0, 12.0, size=heads)
    return ada, qk_scale


def test_variant_defaults_are_the_base_block_exactly():
    rng = np.random.default_rng(20)
    x, W, kp, vp = _rand_block(rng, B=2, N=9, P=4)
    idx = np.array([[0, 1, 4, 8], [2, 3, 5, 6]])
    base = O.pruned_block(x, idx, W, kp, vp, heads=2)
    neutral = np.zeros((2, 6, 8)); neutral[:, 2] = 1.0; neutral[:, 5] = 1.0
    for got in (O.pruned_block(x, idx, W, kp, vp, heads=2, gelu_form="erf", qk_scale=None, ada=None),
                O.pruned_block(x, idx, W, kp, vp, heads=2, ada=neutral)):
        for a, b in zip(got, base):
            assert np.array_equal(a, b)


def test_gelu_tanh_values_and_library():
    v = np.array([-30.0, -3.0, -1.0, -1e-9, 0.0, 1e-9, 0.5, 1.0, 3.0, 30.0])
    g = O.gelu_tanh(v)
    assert g[4] == 0.0 and g[0] == 0.0 and g[-1] == 30.0
    # x - gelu(x) = gelu(-x) * (-1): the two tails sum to the identity, g(x) - g(-x) = x
    np.testing.assert_allclose(g - O.gelu_tanh(-v), v, rtol=1e-15, atol=1e-300)
    np.testing.assert_allclose(g, F.gelu(torch.from_numpy(v), approximate="tanh").numpy(), rtol=1e-14, atol=1e-300)
    # hand value at 1: 0.5 (1 + tanh(sqrt(2/pi) * 1.044715))
    assert g[7] == pytest.approx(0.5 * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * 1.044715)), rel=1e-15)
    # the two forms differ by at most ~5e-4 in absolute terms and they do differ
    d = np.abs(O.gelu_tanh(np.linspace(-6, 6, 2001)) - O.gelu(np.linspace(-6, 6, 2001)))
    assert 1e-4 < d.max() < 1e-3


def test_variant_gates_and_modulation_reductions():
    rng = np.random.default_rng(21)
    x, W, kp, vp = _rand_block(rng, B=2, N=9, P=4)
    idx = np.array([[0, 1, 4, 8], [2, 3, 5, 6]])
    ada, _ = _rand_variant(rng, 2, 8, 2)
    xs = np.stack([x[b, idx[b]] for b in range(2)])
    # both gates 0: the block is the identity on the kept rows; K/V rows still come from the modulated norm
    a0 = ada.copy(); a0[:, 2] = 0.0; a0[:, 5] = 0.0
    y, kn, vn = O.pruned_block(x, idx, W, kp, vp, heads=2, ada=a0)
    assert np.array_equal(y, xs)
    for b in range(2):
        u = O.layer_norm(xs[b]) * (1.0 + a0[b, 1]) + a0[b, 0]
        qkv = u @ W["w_qkv"].T + W["b_qkv"]
        np.testing.assert_allclose(kn[b], qkv[:, 8:16], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(vn[b], qkv[:, 16:], rtol=1e-12, atol=1e-14)
    # the output is affine in each gate with the other parts fixed: gate2 enters only the last step
    y1 = O.pruned_block(x, idx, W, kp, vp, heads=2, ada=ada)[0]
    a2 = ada.copy(); a2[:, 5] *= 3.0
    y3 = O.pruned_block(x, idx, W, kp, vp, heads=2, ada=a2)[0]
    a_off = ada.copy(); a_off[:, 5] = 0.0
    x1 = O.pruned_block(x, idx, W, kp, vp, heads=2, ada=a_off)[0]            # gate2 = 0 leaves x1
    np.testing.assert_allclose(y3 - x1, 3.0 * (y1 - x1), rtol=1e-10, atol=1e-12)
    # scale = -1 wipes the normalised input: with shift s the projections see the constant row s
    a3 = ada.copy(); a3[:, 1] = -1.0
    _, kn, _ = O.pruned_block(x, idx, W, kp, vp, heads=2, ada=a3)
    for b in range(2):
        ref = a3[b, 0] @ W["w_qkv"][8:16].T + W["b_qkv"][8:16]
        np.testing.assert_allclose(kn[b], np.tile(ref, (4, 1)), rtol=1e-12, atol=1e-14)
    # image b is modulated by ada[b] only
    a4 = ada.copy(); a4[1] = rng.standard_normal((6, 8))
    y4 = O.pruned_block(x, idx, W, kp, vp, heads=2, ada=a4)[0]
    assert np.array_equal(y4[0], y1[0]) and not np.allclose(y4[1], y1[1])


def test_variant_unit_length_queries_and_keys():
    rng = np.random.default_rng(22)
    x, W, kp, vp = _rand_block(rng, B=1, N=8, C=8, heads=2, P=3)
    idx = np.array([[1, 2, 5, 7]])
    qk_scale = np.array([4.0, 9.0])
    kp = np.concatenate([O.unit_rows(kp[..., :4]), O.unit_rows(kp[..., 4:])], axis=-1)   # the cache holds unit keys
    y, kn, vn = O.pruned_block(x, idx, W, kp, vp, heads=2, qk_scale=qk_scale)
    for h in range(2):
        np.testing.assert_allclose(np.linalg.norm(kn[0][:, h * 4:(h + 1) * 4], axis=-1), 1.0, rtol=1e-14)
    # a positive rescaling of a head's query projection, or of its key projection, changes nothing
    W2 = {n: (None if a is None else a.copy()) for n, a in W.items()}
    W2["w_qkv"][0:4] *= 7.0; W2["b_qkv"][0:4] *= 7.0            # head 0 queries
    W2["w_qkv"][12:16] *= 0.2; W2["b_qkv"][12:16] *= 0.2        # head 1 keys
    y2, kn2, _ = O.pruned_block(x, idx, W2, kp, vp, heads=2, qk_scale=qk_scale)
    np.testing.assert_allclose(y2, y, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(kn2, kn, rtol=1e-12, atol=1e-14)
    # multiplier 0: every score is 0, attention is the plain mean of all value rows
    y0, _, vn0 = O.pruned_block(x, idx, W, kp, vp, heads=2, qk_scale=np.zeros(2))
    vmean = np.concatenate([vp[0], vn0[0]]).mean(axis=0)
    xs = x[0, idx[0]]
    x1 = xs + vmean @ W["w_o"].T + W["b_o"]
    ref = x1 + O.gelu(O.layer_norm(x1) @ W["w_fc1"].T + W["b_fc1"]) @ W["w_fc2"].T + W["b_fc2"]
    np.testing.assert_allclose(y0[0], ref, rtol=1e-11, atol=1e-13)
    # a zero key row stays zero (no division by zero)
    assert np.array_equal(O.unit_rows(np.zeros((2, 4))), np.zeros((2, 4)))


@pytest.mark.parametrize("use_ada,use_qk,form", [(True, False, "erf"), (False, True, "erf"), (False, False, "tanh"),
                                                 (True, True, "tanh")])
def test_variant_library_second_opinion_torch_float64(use_ada, use_qk, form):
    rng = np.random.default_rng(23)
    C, heads, dh = 16, 4, 4
    x, W, kp, vp = _rand_block(rng, B=2, N=12, C=C, heads=heads, P=5)
    idx = np.array([[0, 2, 3, 7, 10, 11], [1, 2, 4, 5, 6, 9]])
    ada, qk_scale = _rand_variant(rng, 2, C, heads)
    if use_qk:
        kp = O.unit_rows(kp.reshape(2, 5, heads, dh)).reshape(2, 5, C)
    y, kn, vn = O.pruned_block(x, idx, W, kp, vp, heads=heads, gelu_form=form,
                               qk_scale=qk_scale if use_qk else None, ada=ada if use_ada else None)
    t = {n: torch.from_numpy(a) for n, a in W.items()}
    hd = lambda a: a.reshape(a.shape[0], heads, dh).transpose(0, 1)          # [heads, rows, dh]
    for b in range(2):
        m = [torch.from_numpy(v) for v in ada[b]] if use_ada else [0.0, 0.0, 1.0, 0.0, 0.0, 1.0]
        xs = torch.from_numpy(x[b, idx[b]])
        u = torch.addcmul(m[0] + F.layer_norm(xs, (C,), eps=1e-6), F.layer_norm(xs, (C,), eps=1e-6), torch.as_tensor(m[1])) \
            if use_ada else F.layer_norm(xs, (C,), eps=1e-6)
        qkv = F.linear(u, t["w_qkv"], t["b_qkv"])
        q, kk, vv = qkv.split(C, dim=-1)
        qh, kh = hd(q), hd(kk)
        if use_qk:
            qh = F.normalize(qh, dim=-1) * torch.from_numpy(qk_scale)[:, None, None]
            kh = F.normalize(kh, dim=-1)
        K = torch.cat([hd(torch.from_numpy(kp[b])), kh], dim=1)
        V = torch.cat([torch.from_numpy(vp[b]), vv])
        a = F.scaled_dot_product_attention(qh, K, hd(V), scale=1.0 if use_qk else None)
        a = a.transpose(0, 1).reshape(-1, C)
        x1 = xs + m[2] * F.linear(a, t["w_o"], t["b_o"])
        n2 = F.layer_norm(x1, (C,), eps=1e-6)
        if use_ada:
            n2 = n2 * (1.0 + m[4]) + m[3]
        hdn = F.gelu(F.linear(n2, t["w_fc1"], t["b_fc1"]), approximate="tanh" if form == "tanh" else "none")
        ref = x1 + m[5] * F.linear(hdn, t["w_fc2"], t["b_fc2"])
        np.testing.assert_allclose(y[b], ref.numpy(), rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(kn[b], kh.transpose(0, 1).reshape(-1, C).numpy(), rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(vn[b], vv.numpy(), rtol=1e-10, atol=1e-12)


# ---- other interpolation kernels for the residual cache -------------------------------------
def test_nearest_upsample_pins():
    rng = np.random.default_rng(30)
    c = rng.standard_normal((2, 12, 3))
    assert np.array_equal(O.nearest_upsample(c, 3, 4, 3, 4), c)                       # same grid: identity
    # integer factor: every source cell is repeated as a 2 x 3 patch
    up = O.nearest_upsample(c, 3, 4, 6, 12).reshape(2, 6, 12, 3)
    src = c.reshape(2, 3, 4, 3)
    assert np.array_equal(up, np.repeat(np.repeat(src, 2, axis=1), 3, axis=2))
    # hand case 1 x 3 -> 1 x 5: centres 0.3, 0.9, 1.5, 2.1, 2.7 fall in cells 0, 0, 1, 2, 2
    row = np.array([10.0, 20.0, 30.0]).reshape(1, 3, 1)
    assert O.nearest_upsample(row, 1, 3, 1, 5).ravel().tolist() == [10.0, 10.0, 20.0, 30.0, 30.0]
    # downsampling picks, never mixes
    down = O.nearest_upsample(c, 3, 4, 2, 2)
    assert all(any(np.array_equal(v, s) for s in c[0]) for v in down[0])


@pytest.mark.parametrize("hp,wp,h,w", [(13, 13, 16, 16), (3, 5, 7, 6), (48, 48, 64, 64), (5, 5, 4, 4), (1, 1, 3, 2)])
def test_nearest_and_bicubic_library_second_opinion(hp, wp, h, w):
    rng = np.random.default_rng(31)
    c = rng.standard_normal((2, hp * wp, 3))
    t = torch.from_numpy(c).reshape(2, hp, wp, 3).permute(0, 3, 1, 2)
    back = lambda r: r.permute(0, 2, 3, 1).reshape(2, h * w, 3).numpy()
    ref_n = F.interpolate(t, size=(h, w), mode="nearest-exact")
    assert np.array_equal(O.nearest_upsample(c, hp, wp, h, w), back(ref_n))
    ref_c = F.interpolate(t, size=(h, w), mode="bicubic", align_corners=False, antialias=False)
    np.testing.assert_allclose(O.bicubic_upsample(c, hp, wp, h, w), back(ref_c), rtol=1e-12, atol=1e-13)


def test_bicubic_upsample_closed_forms(monkeypatch):
    rng = np.random.default_rng(32)
    c = rng.standard_normal((2, 12, 3))
    np.testing.assert_allclose(O.bicubic_upsample(c, 3, 4, 3, 4), c, atol=1e-15)       # same grid: weights (0, 1, 0, 0)
    const = np.full((1, 6, 2), 2.5)
    np.testing.assert_allclose(O.bicubic_upsample(const, 2, 3, 5, 7), 2.5, rtol=1e-14)  # the weights sum to 1
    # weights at t = 1/2 with a = -3/4: (-3/32, 19/32, 19/32, -3/32)
    np.testing.assert_allclose(O._cubic_weights(np.array([0.5]))[0], [-3 / 32, 19 / 32, 19 / 32, -3 / 32], rtol=1e-15)
    np.testing.assert_allclose(O._cubic_weights(np.linspace(0, 0.999, 50)).sum(axis=-1), 1.0, rtol=1e-14)
    # 1 x 4 -> 1 x 8: output 3 sits at src 1.25 (taps 0..3, t = 0.25); by hand from the kernel polynomials
    row = np.array([1.0, -2.0, 4.0, 0.5]).reshape(1, 4, 1)
    up = O.bicubic_upsample(row, 1, 4, 1, 8).ravel()
    t = 0.25
    near = lambda d: (1.25 * d - 2.25) * d * d + 1.0
    far = lambda d: ((-0.75 * d + 3.75) * d - 6.0) * d + 3.0
    want = far(1 + t) * 1.0 + near(t) * -2.0 + near(1 - t) * 4.0 + far(2 - t) * 0.5
    assert up[3] == pytest.approx(want, rel=1e-14)
    # the first output sits at src -0.25: floor -1, t = 0.75, taps -2..1 clamped to (0, 0, 0, 1)
    t = 0.75
    want0 = (far(1 + t) + near(t) + near(1 - t)) * 1.0 + far(2 - t) * -2.0
    assert up[0] == pytest.approx(want0, rel=1e-14)
    # the same polynomials with a = -1/2 have a vanishing first moment: linear ramps are then reproduced in
    # the interior (with a = -3/4 they are not, which the library comparison above covers)
    monkeypatch.setattr(O, "CUBIC_A", -0.5)
    hp = wp = 13; h = w = 16
    yy, xx = np.meshgrid(np.arange(hp), np.arange(wp), indexing="ij")
    ramp = (2.0 * yy - 3.0 * xx + 1.0).reshape(1, hp * wp, 1)
    got = O.bicubic_upsample(ramp, hp, wp, h, w).reshape(h, w)
    sy = (np.arange(h) + 0.5) * hp / h - 0.5
    inside = (sy >= 1) & (sy <= hp - 2)
    ref = 2.0 * sy[:, None] - 3.0 * sy[None, :] + 1.0
    sel = np.ix_(inside, inside)
    np.testing.assert_allclose(got[sel], ref[sel], rtol=1e-12, atol=1e-12)
    monkeypatch.setattr(O, "CUBIC_A", -0.75)
    assert not np.allclose(O.bicubic_upsample(ramp, hp, wp, h, w).reshape(h, w)[sel], ref[sel], atol=1e-3)
    # transposed field -> transposed result
    f = rng.standard_normal((5, 7))
    a = O.bicubic_upsample(f.reshape(1, -1, 1), 5, 7, 8, 9).reshape(8, 9)
    b = O.bicubic_upsample(f.T.reshape(1, -1, 1), 7, 5, 9, 8).reshape(9, 8)
    np.testing.assert_allclose(a, b.T, rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("interp", ["nearest", "bicubic"])
def test_merge_rules_with_other_interpolation(interp):
    rng = np.random.default_rng(33)
    B, hp, wp, h, w, C = 2, 3, 3, 4, 4, 5
    x = rng.standard_normal((B, h * w, C))
    cache_prev = rng.standard_normal((B, hp * wp, C))
    idx = np.array([[0, 5, 6, 15], [2, 3, 9, 10]])
    y = rng.standard_normal((B, 4, C))
    out, cn = O.merge_cache(x, y, idx, cache_prev, hp, wp, h, w, interp=interp)
    up = O.UPSAMPLERS[interp](cache_prev, hp, wp, h, w)
    base, _ = O.merge_cache(x, y, idx, cache_prev, hp, wp, h, w)
    for b in range(B):
        kept = idx[b]
        pruned = np.setdiff1d(np.arange(h * w), kept)
        assert np.array_equal(out[b, kept], y[b]) and np.array_equal(out[b, kept], base[b, kept])
        np.testing.assert_allclose(out[b, pruned], x[b, pruned] + up[b, pruned], atol=1e-15)
        assert not np.allclose(out[b, pruned], base[b, pruned])            # the kernel matters on pruned rows
    np.testing.assert_allclose(cn, out - x, atol=0)


# ---- cross-attention sub-layer ---------------------------------------------------------------
def _rand_cross(rng, B, C, Lt, bias=True):
    return {"w_cq": rng.standard_normal((C, C)) * 0.3, "b_cq": rng.standard_normal(C) * 0.1 if bias else None,
            "w_co": rng.standard_normal((C, C)) * 0.3, "b_co": rng.standard_normal(C) * 0.1 if bias else None,
            "k_text": rng.standard_normal((B, Lt, C)), "v_text": rng.standard_normal((B, Lt, C))}


def test_cross_attention_reductions():
    rng = np.random.default_rng(40)
    x, W, kp, vp = _rand_block(rng, B=2, N=9, P=4)
    idx = np.array([[0, 1, 4, 8], [2, 3, 5, 6]])
    base = O.pruned_block(x, idx, W, kp, vp, heads=2)
    cr = _rand_cross(rng, 2, 8, 5)
    # a zero output projection switches the sub-layer off; K/V rows appended to the self-attention cache never see it
    off = dict(cr, w_co=np.zeros((8, 8)), b_co=None)
    got = O.pruned_block(x, idx, W, kp, vp, heads=2, cross=off)
    for a, b in zip(got, base):
        assert np.array_equal(a, b)
    full = O.pruned_block(x, idx, W, kp, vp, heads=2, cross=cr)
    assert np.array_equal(full[1], base[1]) and np.array_equal(full[2], base[2])
    assert not np.allclose(full[0], base[0])
    # one condition token: every query attends to it alone, so with the FFN output projection zeroed
    # y = x1 + v_text W_co^T + b_co for every kept row
    Wz = dict(W, w_fc2=np.zeros_like(W["w_fc2"]), b_fc2=None)
    one = _rand_cross(rng, 2, 8, 1)
    y1 = O.pruned_block(x, idx, Wz, kp, vp, heads=2, cross=one)[0]
    y0 = O.pruned_block(x, idx, Wz, kp, vp, heads=2)[0]
    for b in range(2):
        want = one["v_text"][b, 0] @ one["w_co"].T + one["b_co"]
        np.testing.assert_allclose(y1[b] - y0[b], np.tile(want, (4, 1)), rtol=1e-11, atol=1e-13)
    # the order of the condition tokens does not matter; image b reads its own tokens only
    perm = np.array([3, 0, 4, 1, 2])
    shuffled = dict(cr, k_text=cr["k_text"][:, perm], v_text=cr["v_text"][:, perm])
    np.testing.assert_allclose(O.pruned_block(x, idx, W, kp, vp, heads=2, cross=shuffled)[0], full[0], rtol=1e-11, atol=1e-13)
    other = dict(cr, k_text=cr["k_text"].copy(), v_text=cr["v_text"].copy())
    other["v_text"][1] += 1.0
    y_other = O.pruned_block(x, idx, W, kp, vp, heads=2, cross=other)[0]
    assert np.array_equal(y_other[0], full[0][0]) and not np.allclose(y_other[1], full[0][1])
    # identical keys: uniform attention, the output is the mean value row
    same = dict(cr, k_text=np.tile(cr["k_text"][:, :1], (1, 5, 1)))
    ys = O.pruned_block(x, idx, Wz, kp, vp, heads=2, cross=same)[0]
    for b in range(2):
        want = same["v_text"][b].mean(axis=0) @ same["w_co"].T + same["b_co"]
        np.testing.assert_allclose(ys[b] - y0[b], np.tile(want, (4, 1)), rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("bias,with_others", [(True, False), (False, False), (True, True)])
def test_cross_attention_library_second_opinion_torch_float64(bias, with_others):
    rng = np.random.default_rng(41)
    C, heads, dh, Lt = 16, 4, 4, 7
    x, W, kp, vp = _rand_block(rng, B=2, N=12, C=C, heads=heads, P=5)
    idx = np.array([[0, 2, 3, 7, 10, 11], [1, 2, 4, 5, 6, 9]])
    cr = _rand_cross(rng, 2, C, Lt, bias=bias)
    ada, _ = _rand_variant(rng, 2, C, heads)
    kw = dict(ada=ada, gelu_form="tanh") if with_others else {}
    y, kn, vn = O.pruned_block(x, idx, W, kp, vp, heads=heads, cross=cr, **kw)
    t = {n: torch.from_numpy(a) for n, a in W.items()}
    c = {n: (None if a is None else torch.from_numpy(a)) for n, a in cr.items()}
    hd = lambda a: a.reshape(a.shape[0], heads, dh).transpose(0, 1)
    for b in range(2):
        m = [torch.from_numpy(v) for v in ada[b]] if with_others else [0.0, 0.0, 1.0, 0.0, 0.0, 1.0]
        xs = torch.from_numpy(x[b, idx[b]])
        u = F.layer_norm(xs, (C,), eps=1e-6) * (1.0 + m[1]) + m[0]
        q, kk, vv = F.linear(u, t["w_qkv"], t["b_qkv"]).split(C, dim=-1)
        K = torch.cat([torch.from_numpy(kp[b]), kk])
        V = torch.cat([torch.from_numpy(vp[b]), vv])
        a = F.scaled_dot_product_attention(hd(q), hd(K), hd(V)).transpose(0, 1).reshape(-1, C)
        x1 = xs + m[2] * F.linear(a, t["w_o"], t["b_o"])
        qc = F.linear(F.layer_norm(x1, (C,), eps=1e-6), c["w_cq"], c["b_cq"])
        ac = F.scaled_dot_product_attention(hd(qc), hd(c["k_text"][b]), hd(c["v_text"][b])).transpose(0, 1).reshape(-1, C)
        x1 = x1 + F.linear(ac, c["w_co"], c["b_co"])
        n2 = F.layer_norm(x1, (C,), eps=1e-6) * (1.0 + m[4]) + m[3]
        hdn = F.gelu(F.linear(n2, t["w_fc1"], t["b_fc1"]), approximate="tanh" if with_others else "none")
        ref = x1 + m[5] * F.linear(hdn, t["w_fc2"], t["b_fc2"])
        np.testing.assert_allclose(y[b], ref.numpy(), rtol=1e-9, atol=1e-11)


# ---- per-image keep counts (the reduction ratios are per instance) ---------------------------------------
def _ragged_case(rng):
    B, N, C, P = 3, 7, 8, 4
    x, W, kp, vp = _rand_block(rng, B=B, N=N, C=C, P=P)
    counts = [4, 0, 7]                                   # some, none, all
    kv_rows = [3, 1, 4]                                  # each image's own number of prior rows
    idx = np.full((B, N), -1, dtype=np.int64)
    idx[0, :4] = [1, 2, 4, 6]
    idx[2, :7] = np.arange(7)
    return x, W, kp, vp, idx, counts, kv_rows


def test_per_image_counts_equal_each_image_run_on_its_own():
    """A batch whose images keep different numbers of tokens and hold different numbers of prior rows: every
    image's outputs are those of a single-image call with its own trimmed index list and prior rows."""
    rng = np.random.default_rng(21)
    x, W, kp, vp, idx, counts, kv_rows = _ragged_case(rng)
    y, kn, vn = O.pruned_block(x, idx, W, kp, vp, heads=2, kv_rows=kv_rows)
    assert y.shape == (3, 7, 8)
    for b, (k, P) in enumerate(zip(counts, kv_rows)):
        if k:
            y1, k1, v1 = O.pruned_block(x[b:b + 1], idx[b:b + 1, :k], W, kp[b:b + 1, :P], vp[b:b + 1, :P], heads=2)
            np.testing.assert_allclose(y[b, :k], y1[0], rtol=0, atol=0)
            np.testing.assert_allclose(kn[b, :k], k1[0], rtol=0, atol=0)
            np.testing.assert_allclose(vn[b, :k], v1[0], rtol=0, atol=0)
        assert not y[b, k:].any() and not kn[b, k:].any() and not vn[b, k:].any()
    # image 2 keeps everything: the independent scalar dense block on its own prior rows
    Wl = {n: a.tolist() for n, a in W.items()}
    ref, rk, rv = _dense_block_scalar(x[2].tolist(), Wl, kp[2, :4].tolist(), vp[2, :4].tolist(), 2)
    np.testing.assert_allclose(y[2], np.array(ref), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(kn[2], np.array(rk), rtol=1e-10, atol=1e-12)


def test_per_image_counts_nothing_leaks_between_images_or_from_unused_rows():
    rng = np.random.default_rng(22)
    x, W, kp, vp, idx, counts, kv_rows = _ragged_case(rng)
    y, kn, vn = O.pruned_block(x, idx, W, kp, vp, heads=2, kv_rows=kv_rows)
    # prior rows past an image's own count, and another image's tokens, are never read
    kp2, vp2, x2 = kp.copy(), vp.copy(), x.copy()
    for b, P in enumerate(kv_rows):
        kp2[b, P:] = np.nan
        vp2[b, P:] = np.nan
    x2[1] = np.nan                                       # image 1 keeps nothing: its tokens are never gathered
    y2, kn2, vn2 = O.pruned_block(x2, idx, W, kp2, vp2, heads=2, kv_rows=kv_rows)
    assert np.array_equal(y, y2) and np.array_equal(kn, kn2) and np.array_equal(vn, vn2)
    # uniform counts written with the per-image arguments are the plain call
    full = np.tile(np.arange(5), (3, 1))
    a = O.pruned_block(x, full, W, kp, vp, heads=2)
    b_ = O.pruned_block(x, full, W, kp, vp, heads=2, kv_rows=[4, 4, 4])
    for u, v in zip(a, b_):
        assert np.array_equal(u, v)
    with pytest.raises(AssertionError):
        O.pruned_block(x, np.array([[0, -1, 3]] * 3), W, kp, vp, heads=2)      # a hole is not a tail


def test_merge_with_per_image_counts():
    rng = np.random.default_rng(23)
    B, hp, wp, h, w, C = 3, 3, 3, 4, 4, 5
    N = h * w
    x = rng.standard_normal((B, N, C))
    cache_prev = rng.standard_normal((B, hp * wp, C))
    counts = [3, 0, N]
    idx = np.full((B, N), -1, dtype=np.int64)
    idx[0, :3] = [2, 7, 11]
    idx[2] = np.arange(N)
    y = rng.standard_normal((B, N, C))
    for b, k in enumerate(counts):
        y[b, k:] = np.nan                                # rows behind an image's count must never be used
    out, cn = O.merge_cache(x, y, idx, cache_prev, hp, wp, h, w)
    assert np.isfinite(out).all() and np.isfinite(cn).all()
    for b, k in enumerate(counts):
        o1, c1 = O.merge_cache(x[b:b + 1], y[b:b + 1, :k], idx[b:b + 1, :k], cache_prev[b:b + 1], hp, wp, h, w)
        assert np.array_equal(out[b], o1[0]) and np.array_equal(cn[b], c1[0])
    up = O.bilinear_upsample(cache_prev, hp, wp, h, w)
    np.testing.assert_allclose(out[1], x[1] + up[1], atol=0)           # nothing kept: everything from the cache
    assert np.array_equal(out[2], y[2])                                 # everything kept
