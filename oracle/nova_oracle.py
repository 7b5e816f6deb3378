"""CPU oracle for the entropy-pruned transformer block (TEST INFRASTRUCTURE ONLY).

A plain, slow, float64 NumPy statement of what the hot path computes, written
from the paper's definitions.  It shares no code with the HIP path and must
never be imported by the product package: only tests, the smoke check and the
benchmark's cpu_baseline leg may call it.

What each function follows:
  entropy, mean_entropy   -- token predictive entropy (Sec. 3.3, "Adaptive
                             Acceleration Activation", the entropy equation and
                             the scale-mean equation); natural logarithm.
  head_entropy            -- the same entropy taken straight from a linear head's input
                             (Sec. 4, "Entropy Computation Overhead": the distributions are
                             the ones decoding produces anyway).
  bitwise_entropy         -- the entropy equation for a head that predicts a token as d
                             independent bits (the Infinity backbone of Sec. 4): the sum of
                             the bits' binary entropies.  This factorised form is this
                             build's reading; the paper prints only the categorical one.
  select                  -- "pruning low-entropy tokens according to the token
                             reduction ratio" (Sec. 3.3, Dual-Linkage Acceleration,
                             last sentence) / "maintaining highest-entropy tokens"
                             (Sec. 3.2): the k largest entropies are kept.
  pruned_block            -- Layer_j applied to the kept tokens only (Sec. 3.3,
                             Residual Cache Reuse, first equation).  The paper
                             leaves Layer_j opaque; the block computed here is this
                             build's definition (pre-norm, affine-free LayerNorm,
                             eps 1e-6, erf GELU, softmax scale 1/sqrt(dh), biases).
                             Beyond the special cases tested (k = N equals a dense
                             block, permutation equivariance, degenerate weights,
                             library second opinions) its parity is unpinned
                             against the paper.
  pruned_block(variants)  -- the same block as the backbones of Sec. 4 build it: modulation of
                             both norms and gating of both branches by per-image vectors
                             (adaptive LayerNorm conditioning), unit-length queries and keys
                             per head with a per-head score multiplier in place of 1/sqrt(dh),
                             tanh-form GELU, a cross-attention sub-layer over condition tokens.  The paper names the backbones, not these
                             details; the formulas are this build's reading (parity unpinned
                             against the paper; pinned to reductions to the base block,
                             invariances and library second opinions).
  bilinear_upsample,
  merge_cache             -- Cache_{t,j} = R_out - R_in, its interpolation to the
                             next grid and the reuse rule for pruned tokens (Sec. 3.3,
                             Residual Cache Reuse, second and third equations).
  nearest_upsample,
  bicubic_upsample        -- other interpolation kernels for the same step (the paper says
                             only that the cache is interpolated): nearest cell, and cubic
                             convolution with a = -0.75 as image libraries define it.

Readings taken where the paper is silent are listed in the repository's design
notes; the ones that matter here: ties in entropy keep the lower index; NaN
entropies rank below every number; the cache after a pruned scale is
out - in at every position; interpolation is bilinear with half-pixel centres.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf

LN_EPS = 1e-6


# ----------------------------------------------------------------------------
# entropy
# ----------------------------------------------------------------------------
def entropy(logits: np.ndarray) -> np.ndarray:
    """H_i = -sum_v p_i(v) ln p_i(v), p_i = softmax(logits_i); any leading shape, last axis V."""
    x = np.asarray(logits, dtype=np.float64)
    m = np.max(x, axis=-1, keepdims=True)
    e = np.exp(x - m)
    Z = np.sum(e, axis=-1, keepdims=True)
    p = e / Z
    # p ln p -> 0 as p -> 0
    with np.errstate(divide="ignore", invalid="ignore"):
        plogp = np.where(p > 0.0, p * np.log(p), 0.0)
    return -np.sum(plogp, axis=-1)


def head_entropy(hidden: np.ndarray, w_head: np.ndarray, b_head=None) -> np.ndarray:
    """Entropy of the distributions a linear prediction head produces: logits = hidden W^T + b
    (W out-feature major, [V, C]), then `entropy` over V.  The paper takes the distributions
    from standard decoding (Sec. 4, "Entropy Computation Overhead"); this is that composition."""
    logits = _f64(hidden) @ _f64(w_head).T
    if b_head is not None:
        logits = logits + _f64(b_head)
    return entropy(logits)


def bitwise_entropy(bit_logits: np.ndarray) -> np.ndarray:
    """Token entropy of a bitwise token head: the token is d independent binary choices, bit i with
    the two logits bit_logits[..., i, 0:2], so the token's entropy is the sum of the d binary
    entropies (the entropy equation of Sec. 3.3 applied to a product distribution).  [..., d, 2] -> [...]."""
    x = np.asarray(bit_logits, dtype=np.float64)
    assert x.shape[-1] == 2
    return np.sum(entropy(x), axis=-1)


def mean_entropy(H: np.ndarray) -> np.ndarray:
    """Scale mean entropy: arithmetic mean over the N tokens of each batch row."""
    H = np.asarray(H, dtype=np.float64)
    return np.sum(H, axis=-1) / H.shape[-1]


# ----------------------------------------------------------------------------
# selection
# ----------------------------------------------------------------------------
def select(H32: np.ndarray, k) -> tuple[np.ndarray, np.ndarray]:
    """Keep the k highest-entropy tokens of every batch row.

    H32: [B, N] float32 entropies (compared as float32 numbers, -0 == +0).
    k: int or length-B sequence.  Order: entropy descending, then index
    ascending; NaN ranks below every number.  Returns (idx [B, kmax] int32,
    ascending, unused tail = -1; mask [B, N] uint8).
    """
    H32 = np.asarray(H32, dtype=np.float32)
    B, N = H32.shape
    ks = np.full(B, k, dtype=np.int64) if np.isscalar(k) else np.asarray(k, dtype=np.int64)
    assert ks.shape == (B,) and np.all(ks >= 0) and np.all(ks <= N)
    kmax = int(ks.max()) if B else 0
    idx = np.full((B, kmax), -1, dtype=np.int32)
    mask = np.zeros((B, N), dtype=np.uint8)
    index = np.arange(N)
    for b in range(B):
        h = H32[b]
        isnan = np.isnan(h)
        neg = np.where(isnan, 0.0, -h.astype(np.float64))
        # lexsort: last key is primary.  NaNs last, then larger entropy first, then lower index.
        order = np.lexsort((index, neg, isnan))
        kept = np.sort(order[: ks[b]])
        idx[b, : ks[b]] = kept
        mask[b, kept] = 1
    return idx, mask


# ----------------------------------------------------------------------------
# the block
# ----------------------------------------------------------------------------
def layer_norm(x: np.ndarray) -> np.ndarray:
    """LayerNorm over the last axis, no affine, biased variance, eps = 1e-6."""
    mu = np.mean(x, axis=-1, keepdims=True)
    var = np.mean((x - mu) ** 2, axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + LN_EPS)


def gelu(x: np.ndarray) -> np.ndarray:
    """Exact (erf) GELU."""
    return 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))


def gelu_tanh(x: np.ndarray) -> np.ndarray:
    """tanh-form GELU: 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3)))."""
    return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))


QK_NORM_EPS = 1e-12


def unit_rows(a: np.ndarray) -> np.ndarray:
    """Rows scaled to unit Euclidean length (a zero row stays zero: the divisor is floored at 1e-12)."""
    n = np.sqrt(np.sum(a * a, axis=-1, keepdims=True))
    return a / np.maximum(n, QK_NORM_EPS)


def softmax(s: np.ndarray) -> np.ndarray:
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def _f64(a):
    return None if a is None else np.asarray(a, dtype=np.float64)


def pruned_block(x, idx, weights, k_prior, v_prior, heads, gelu_form="erf", qk_scale=None, ada=None, cross=None,
                 kv_rows=None):
    """One transformer block on the kept tokens only.

    Per-image keep counts (the reduction ratios of Sec. 3.3, "Dual-Linkage Acceleration", are per
    instance): image b keeps the tokens idx[b, :k_b], where k_b is the number of non-negative entries at
    the front of idx[b] (the unused tail of a row is -1, as `select` writes it), and attends to its own
    kv_rows[b] prior rows (all of k_prior[b] when kv_rows is None) plus its own k_b kept rows.  Every image
    is computed on its own: nothing of one image enters another's result.  Rows past k_b of the three
    outputs are zero.

    Variants (all off by default):
      gelu_form  "erf" | "tanh"
      qk_scale   [heads] or None.  When given, the query and key of every head are scaled to unit
                 length, the scores are qk_scale[h] * <q^, k^> (no 1/sqrt(dh)), and the rows appended
                 to the key cache are the unit-length keys (k_prior already holds such rows).
      ada        [B, 6, C] or None: per-image (shift1, scale1, gate1, shift2, scale2, gate2).
                 u = LN(xs) (1 + scale1) + shift1,  x1 = xs + gate1 * attn_branch,
                 FFN input = LN(x1) (1 + scale2) + shift2,  y = x1 + gate2 * ffn_branch.
      cross      dict or None: a cross-attention sub-layer between the self-attention and the FFN branch,
                 x1 <- x1 + softmax((LN(x1) w_cq^T + b_cq) Kt^T / sqrt(dh)) Vt w_co^T + b_co per head, with
                 "k_text", "v_text" [B, Lt, C] the (already projected) keys / values of the condition tokens
                 and "w_cq", "b_cq", "w_co", "b_co" the query and output projections ([C, C], [C]).

    x        [B, N, C]   block input (all tokens of the current scale)
    idx      [B, k]      kept token indices per batch row
    weights  dict: w_qkv [3C, C], b_qkv [3C], w_o [C, C], b_o [C], w_fc1 [F, C],
             b_fc1 [F], w_fc2 [C, F], b_fc2 [C]  (out-feature major; biases may be None)
    k_prior, v_prior [B, P, C]  keys / values of all prior scales
    Returns y_kept [B, k, C], k_new [B, k, C], v_new [B, k, C] (the rows appended
    to the caches at positions P .. P+k-1, in the order of idx).
    """
    x = _f64(x)
    idx = np.asarray(idx, dtype=np.int64)
    W = {n: _f64(a) for n, a in weights.items()}
    k_prior, v_prior = _f64(k_prior), _f64(v_prior)
    B, N, C = x.shape
    k = idx.shape[1]
    dh = C // heads
    assert dh * heads == C

    def bias(name):
        b = W.get(name)
        return 0.0 if b is None else b

    act = {"erf": gelu, "tanh": gelu_tanh}[gelu_form]
    qk_scale = _f64(qk_scale)
    ada = _f64(ada)
    y_kept = np.zeros((B, k, C))
    k_new = np.zeros((B, k, C))
    v_new = np.zeros((B, k, C))
    k_pitch = k
    for b in range(B):
        if ada is None:
            shift1 = scale1 = shift2 = scale2 = 0.0
            gate1 = gate2 = 1.0
        else:
            shift1, scale1, gate1, shift2, scale2, gate2 = ada[b]
        k = _row_count(idx[b])                            # this image's keep count
        if k == 0:
            continue
        Pb = k_prior.shape[1] if kv_rows is None else int(kv_rows[b])
        xs = x[b, idx[b, :k]]                             # gather kept rows  [k, C]
        u = layer_norm(xs) * (1.0 + scale1) + shift1
        qkv = u @ W["w_qkv"].T + bias("b_qkv")
        q, kk, vv = qkv[:, :C].copy(), qkv[:, C:2 * C].copy(), qkv[:, 2 * C:]
        if qk_scale is not None:
            for h in range(heads):
                sl = slice(h * dh, (h + 1) * dh)
                q[:, sl] = unit_rows(q[:, sl])
                kk[:, sl] = unit_rows(kk[:, sl])
        k_new[b, :k], v_new[b, :k] = kk, vv
        Kc = np.concatenate([k_prior[b, :Pb], kk], axis=0)     # [P + k, C]
        Vc = np.concatenate([v_prior[b, :Pb], vv], axis=0)
        a = np.zeros((k, C))
        for h in range(heads):
            sl = slice(h * dh, (h + 1) * dh)
            scores = q[:, sl] @ Kc[:, sl].T                   # [k, P + k], no mask inside the step
            scores = scores / np.sqrt(dh) if qk_scale is None else scores * qk_scale[h]
            a[:, sl] = softmax(scores) @ Vc[:, sl]
        x1 = xs + gate1 * (a @ W["w_o"].T + bias("b_o"))
        if cross is not None:
            Kt, Vt = _f64(cross["k_text"])[b], _f64(cross["v_text"])[b]
            b_cq = 0.0 if cross.get("b_cq") is None else _f64(cross["b_cq"])
            b_co = 0.0 if cross.get("b_co") is None else _f64(cross["b_co"])
            qc = layer_norm(x1) @ _f64(cross["w_cq"]).T + b_cq
            ac = np.zeros((k, C))
            for h in range(heads):
                sl = slice(h * dh, (h + 1) * dh)
                ac[:, sl] = softmax((qc[:, sl] @ Kt[:, sl].T) / np.sqrt(dh)) @ Vt[:, sl]
            x1 = x1 + ac @ _f64(cross["w_co"]).T + b_co
        hdn = act((layer_norm(x1) * (1.0 + scale2) + shift2) @ W["w_fc1"].T + bias("b_fc1"))
        y_kept[b, :k] = x1 + gate2 * (hdn @ W["w_fc2"].T + bias("b_fc2"))
    assert y_kept.shape[1] == k_pitch
    return y_kept, k_new, v_new


def _row_count(idx_row) -> int:
    """Entries of a kept-index row in front of its -1 tail (all of them when there is no tail)."""
    neg = np.flatnonzero(np.asarray(idx_row) < 0)
    n = int(neg[0]) if neg.size else len(idx_row)
    assert np.all(np.asarray(idx_row)[n:] < 0), "a -1 tail must be contiguous"
    return n


# ----------------------------------------------------------------------------
# residual cache reuse
# ----------------------------------------------------------------------------
def _axis_taps(n_in: int, n_out: int):
    """Half-pixel-centre linear interpolation taps along one axis."""
    dst = np.arange(n_out, dtype=np.float64)
    src = (dst + 0.5) * (n_in / n_out) - 0.5
    src = np.maximum(src, 0.0)
    i0 = np.minimum(np.floor(src).astype(np.int64), n_in - 1)
    i1 = np.minimum(i0 + 1, n_in - 1)
    w1 = src - i0
    return i0, i1, w1


def bilinear_upsample(cache_prev, hp: int, wp: int, h: int, w: int) -> np.ndarray:
    """[B, hp*wp, C] on the prior grid -> [B, h*w, C] on the current grid."""
    c = _f64(cache_prev)
    B, _, C = c.shape
    c = c.reshape(B, hp, wp, C)
    y0, y1, wy = _axis_taps(hp, h)
    x0, x1, wx = _axis_taps(wp, w)
    rows = c[:, y0] * (1.0 - wy)[None, :, None, None] + c[:, y1] * wy[None, :, None, None]   # [B, h, wp, C]
    out = rows[:, :, x0] * (1.0 - wx)[None, None, :, None] + rows[:, :, x1] * wx[None, None, :, None]
    return out.reshape(B, h * w, C)


def nearest_upsample(cache_prev, hp: int, wp: int, h: int, w: int) -> np.ndarray:
    """Nearest source cell of each output cell centre: index min(floor((dst + 0.5) n_in / n_out), n_in - 1),
    evaluated in integers ((2 dst + 1) n_in // (2 n_out)) so that centres on a cell boundary are exact."""
    c = _f64(cache_prev)
    B, _, C = c.shape
    c = c.reshape(B, hp, wp, C)
    iy = np.minimum(((2 * np.arange(h, dtype=np.int64) + 1) * hp) // (2 * h), hp - 1)
    ix = np.minimum(((2 * np.arange(w, dtype=np.int64) + 1) * wp) // (2 * w), wp - 1)
    return c[:, iy][:, :, ix].reshape(B, h * w, C)


CUBIC_A = -0.75


def _cubic_weights(t: np.ndarray) -> np.ndarray:
    """Cubic convolution weights (kernel parameter a = -0.75) of the four taps at offsets -1, 0, 1, 2
    from floor(src), for the fractional position t in [0, 1).  [len(t), 4]."""
    a = CUBIC_A

    def near(d):    # |d| <= 1
        return ((a + 2.0) * d - (a + 3.0)) * d * d + 1.0

    def far(d):     # 1 < |d| < 2
        return ((a * d - 5.0 * a) * d + 8.0 * a) * d - 4.0 * a

    return np.stack([far(t + 1.0), near(t), near(1.0 - t), far(2.0 - t)], axis=-1)


def bicubic_upsample(cache_prev, hp: int, wp: int, h: int, w: int) -> np.ndarray:
    """Separable cubic convolution, half-pixel centres, taps clamped to the grid (edge cells repeat)."""
    c = _f64(cache_prev)
    B, _, C = c.shape
    c = c.reshape(B, hp, wp, C)

    def axis(n_in, n_out):
        src = (np.arange(n_out) + 0.5) * (n_in / n_out) - 0.5
        i0 = np.floor(src).astype(np.int64)
        taps = np.clip(i0[:, None] + np.arange(-1, 3)[None, :], 0, n_in - 1)       # [n_out, 4]
        return taps, _cubic_weights(src - i0)

    ty, wy = axis(hp, h)
    tx, wx = axis(wp, w)
    rows = np.zeros((B, h, wp, C))
    for j in range(4):
        rows += c[:, ty[:, j]] * wy[:, j][None, :, None, None]
    out = np.zeros((B, h, w, C))
    for j in range(4):
        out += rows[:, :, tx[:, j]] * wx[:, j][None, None, :, None]
    return out.reshape(B, h * w, C)


UPSAMPLERS = {"bilinear": bilinear_upsample, "nearest": nearest_upsample, "bicubic": bicubic_upsample}


def merge_cache(x, y_kept, idx, cache_prev, hp, wp, h, w, interp="bilinear"):
    """Scatter kept outputs back; pruned rows reuse the upsampled residual cache.

    interp: "bilinear" (this build's reading of the interpolation), or the variants "nearest", "bicubic".

    out[b, i]       = y_kept[b, s]               if i == idx[b, s]
                    = x[b, i] + cache_up[b, i]   otherwise
    cache_new[b, i] = out[b, i] - x[b, i]
    cache_prev may be None when every token is kept.  Per-image keep counts: a row of idx may end in a
    tail of -1 entries (its image keeps fewer tokens than the row is long); those entries and the rows of
    y_kept that go with them are ignored.
    """
    x, y_kept = _f64(x), _f64(y_kept)
    idx = np.asarray(idx, dtype=np.int64)
    B, N, C = x.shape
    assert N == h * w
    counts = [_row_count(idx[b]) for b in range(B)]
    if min(counts, default=N) < N:
        out = x + UPSAMPLERS[interp](cache_prev, hp, wp, h, w)
    else:
        out = np.zeros_like(x)
    for b in range(B):
        out[b, idx[b, :counts[b]]] = y_kept[b, :counts[b]]
    cache_new = out - x
    return out, cache_new
