"""Pins for the oracle's entropy and selection (CPU only).

Entropy is pinned to closed forms and invariants of the definition (Sec. 3.3,
entropy equation); selection to a brute-force rank count that shares no code
with the oracle's sort (Sec. 3.3, last sentence of Dual-Linkage Acceleration:
the lowest-entropy tokens are pruned).
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import nova_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "entropy_closed_forms.txt")


def _golden_rows():
    rows = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        case, V, m, a, H = line.split()
        rows.append((case, int(V), int(m), float(a), float(H)))
    return rows


@pytest.mark.parametrize("case,V,m,a,H", _golden_rows())
def test_entropy_closed_forms(case, V, m, a, H):
    x = np.zeros(V)
    if case == "twolevel":
        # put the m high logits at scattered positions
        pos = (np.arange(m) * 37) % V
        assert len(set(pos.tolist())) == m
        x[pos] = a
    got = O.entropy(x[None, :])[0]
    # the definitional form -sum p ln p loses a few digits when one p is within 1e-5 of 1
    assert got == pytest.approx(H, rel=1e-10, abs=1e-15)


def test_entropy_uniform_is_lnV_and_onehot_is_zero():
    for V in (2, 7, 512, 4096):
        assert O.entropy(np.full((1, V), 3.25))[0] == pytest.approx(math.log(V), rel=1e-13)
        x = np.full((1, V), -np.inf)
        x[0, V // 3] = 1.5
        assert O.entropy(x)[0] == 0.0
        x = np.zeros((1, V))
        x[0, 0] = 1e4            # one logit far above the rest
        assert O.entropy(x)[0] == 0.0


def test_entropy_invariants():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 300)) * rng.uniform(0.1, 10, size=(5, 1))
    H = O.entropy(x)
    assert np.all(H >= 0) and np.all(H <= math.log(300) + 1e-12)
    # shift invariance, including huge offsets
    for c in (7.0, -1e4, 1e4):
        np.testing.assert_allclose(O.entropy(x + c), H, rtol=1e-9)
    # permutation invariance
    perm = rng.permutation(300)
    np.testing.assert_allclose(O.entropy(x[:, perm]), H, rtol=1e-12)
    # raising the temperature cannot lower the entropy
    taus = [0.25, 0.5, 1.0, 2.0, 4.0, 8.0]
    Ht = np.stack([O.entropy(x / t) for t in taus])
    assert np.all(np.diff(Ht, axis=0) >= -1e-12)


def test_entropy_direct_sum_and_library_second_opinion():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((4, 64)) * 3
    H = O.entropy(x)
    # direct evaluation of -sum p ln p with python floats
    for r in range(4):
        row = [float(v) for v in x[r]]
        Z = sum(math.exp(v) for v in row)
        ref = -sum((math.exp(v) / Z) * math.log(math.exp(v) / Z) for v in row)
        assert H[r] == pytest.approx(ref, rel=1e-12)
    # torch float64: -(softmax * log_softmax).sum
    t = torch.from_numpy(x)
    ref = -(torch.softmax(t, -1) * torch.log_softmax(t, -1)).sum(-1).numpy()
    np.testing.assert_allclose(H, ref, rtol=1e-12)


def test_mean_entropy_is_arithmetic_mean():
    H = np.array([[1.0, 2.0, 6.0], [0.0, 0.0, 3.0]])
    np.testing.assert_allclose(O.mean_entropy(H), [3.0, 1.0])


# ----------------------------------------------------------------------------
# selection
# ----------------------------------------------------------------------------
def _brute_force_kept(h, k):
    """Token i is kept iff fewer than k tokens beat it, where j beats i when
    H_j > H_i, or H_j == H_i and j < i (NaN loses to every number)."""
    n = len(h)
    kept = []
    for i in range(n):
        beats = 0
        for j in range(n):
            if j == i:
                continue
            hi, hj = float(h[i]), float(h[j])
            i_nan, j_nan = math.isnan(hi), math.isnan(hj)
            if i_nan and j_nan:
                better = j < i
            elif i_nan:
                better = True
            elif j_nan:
                better = False
            else:
                better = hj > hi or (hj == hi and j < i)
            beats += better
        if beats < k:
            kept.append(i)
    return kept


@pytest.mark.parametrize("N", [1, 2, 5, 17, 64])
def test_select_matches_brute_force_all_k(N):
    rng = np.random.default_rng(N)
    # few distinct values -> many ties; include +-0 and a NaN on some sizes
    h = rng.choice(np.array([0.0, -0.0, 0.5, 1.25, 3.0, 3.0000002], dtype=np.float32), size=N)
    if N >= 17:
        h[N // 2] = np.nan
    for k in range(N + 1):
        idx, mask = O.select(h[None, :], k)
        kept = _brute_force_kept(h, k)
        assert idx[0, :k].tolist() == kept
        assert mask[0].tolist() == [1 if i in kept else 0 for i in range(N)]


def test_select_random_distinct_and_per_row_k():
    rng = np.random.default_rng(7)
    H = rng.random((3, 40)).astype(np.float32)
    ks = [0, 13, 40]
    idx, mask = O.select(H, ks)
    for b, k in enumerate(ks):
        assert idx[b, :k].tolist() == _brute_force_kept(H[b], k)
        assert int(mask[b].sum()) == k
        assert np.all(idx[b, k:] == -1)


def test_select_all_equal_keeps_lowest_indices():
    H = np.full((2, 33), 1.5, dtype=np.float32)
    idx, mask = O.select(H, 10)
    assert idx.tolist() == [list(range(10))] * 2
    assert mask[:, :10].all() and not mask[:, 10:].any()


def test_select_two_valued_more_ties_than_slots():
    h = np.array([1, 2, 1, 2, 2, 1, 2, 1], dtype=np.float32)[None]
    idx, _ = O.select(h, 3)
    assert idx.tolist() == [[1, 3, 4]]
    idx, _ = O.select(h, 6)
    assert idx.tolist() == [[0, 1, 2, 3, 4, 6]]


def test_select_invariants_large():
    rng = np.random.default_rng(3)
    H = np.round(rng.random((4, 4096)) * 50).astype(np.float32) / 50   # many ties
    k = 1234
    idx, mask = O.select(H, k)
    for b in range(4):
        assert int(mask[b].sum()) == k
        assert np.all(np.diff(idx[b]) > 0)
        assert np.array_equal(np.flatnonzero(mask[b]), idx[b])
        kept, pruned = H[b][mask[b] == 1], H[b][mask[b] == 0]
        thr = kept.min()
        assert thr >= pruned.max()
        tied_kept = np.flatnonzero((H[b] == thr) & (mask[b] == 1))
        tied_pruned = np.flatnonzero((H[b] == thr) & (mask[b] == 0))
        if len(tied_kept) and len(tied_pruned):
            assert tied_kept.max() < tied_pruned.min()


# ---------------------------------------------------------------------------------------------
# entropy straight from a linear head (Sec. 4, "Entropy Computation Overhead")
# ---------------------------------------------------------------------------------------------
def test_head_entropy_special_cases():
    rng = np.random.default_rng(5)
    V, C = 37, 11
    W = rng.standard_normal((V, C))
    # zero hidden state: all logits equal the bias; without a bias the distribution is uniform
    assert np.allclose(O.head_entropy(np.zeros((3, C)), W), np.log(V), rtol=1e-14)
    b = rng.standard_normal(V)
    assert np.allclose(O.head_entropy(np.zeros((2, C)), W, b), O.entropy(b[None, :].repeat(2, 0)), rtol=1e-14)
    # a one-hot hidden state selects one column of W as the logits
    for c in (0, 4, 10):
        h = np.zeros((1, C)); h[0, c] = 1.0
        assert np.allclose(O.head_entropy(h, W), O.entropy(W[:, c][None, :]), rtol=1e-14)
    # adding a constant to every logit (a bias shift) changes nothing
    h = rng.standard_normal((5, C))
    assert np.allclose(O.head_entropy(h, W, b), O.head_entropy(h, W, b + 3.25), rtol=1e-12)


def test_head_entropy_against_scalar_loops():
    rng = np.random.default_rng(6)
    M, V, C = 4, 9, 5
    h, W, b = rng.standard_normal((M, C)), rng.standard_normal((V, C)), rng.standard_normal(V)
    got = O.head_entropy(h, W, b)
    for m in range(M):
        logits = [sum(h[m, c] * W[v, c] for c in range(C)) + b[v] for v in range(V)]
        mx = max(logits)
        Z = sum(math.exp(x - mx) for x in logits)
        H = -sum((math.exp(x - mx) / Z) * ((x - mx) - math.log(Z)) for x in logits)
        assert got[m] == pytest.approx(H, rel=1e-12)


# ---------------------------------------------------------------------------------------------
# bitwise token heads: a token is d independent binary choices
# ---------------------------------------------------------------------------------------------
def test_bitwise_entropy_closed_forms():
    # all bits undecided: d ln 2; all bits certain: 0
    assert np.allclose(O.bitwise_entropy(np.zeros((3, 16, 2))), 16 * math.log(2.0), rtol=1e-15)
    sure = np.zeros((1, 8, 2)); sure[..., 1] = 80.0
    assert O.bitwise_entropy(sure)[0] < 1e-30
    # binary entropy of p = 1/4 on every bit: logit difference ln 3
    x = np.zeros((2, 5, 2)); x[..., 0] = math.log(3.0)
    h = -(0.25 * math.log(0.25) + 0.75 * math.log(0.75))
    assert np.allclose(O.bitwise_entropy(x), 5 * h, rtol=1e-14)


def test_bitwise_entropy_is_the_entropy_of_the_product_distribution():
    # brute force: enumerate all 2^d tokens of the product distribution and apply the categorical equation
    rng = np.random.default_rng(11)
    d = 6
    x = rng.standard_normal((4, d, 2)) * 2.0
    got = O.bitwise_entropy(x)
    for r in range(4):
        p1 = 1.0 / (1.0 + np.exp(x[r, :, 0] - x[r, :, 1]))        # P(bit = 1)
        H = 0.0
        for token in range(1 << d):
            p = 1.0
            for i in range(d):
                p *= p1[i] if (token >> i) & 1 else 1.0 - p1[i]
            H -= p * math.log(p)
        assert got[r] == pytest.approx(H, rel=1e-12)
    # shifting both logits of a bit changes nothing; swapping them changes nothing either
    y = x.copy(); y[:, 2, :] += 1.75; y[:, 4, :] = y[:, 4, ::-1]
    assert np.allclose(O.bitwise_entropy(y), got, rtol=1e-13)
