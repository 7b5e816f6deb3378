"""Entropy straight from a linear head (Sec. 4, "Entropy Computation Overhead") against the oracle's
composition entropy(hidden W^T + b).  Tolerance: the logits are fp32 sums of exact bf16 products
(K <= 2304 terms), so |dH| <= 1e-4 |H| + 1e-5 covers accumulation order and the fp32 softmax sums."""
import math

import numpy as np
import pytest
import torch

import harness as Hn
from oracle import nova_oracle as O


def _case(B, N, C, V, seed, bias=True, wstd=0.05):
    g = torch.Generator().manual_seed(seed)
    hidden = torch.randn(B, N, C, generator=g).to(torch.bfloat16)
    # a spread of row norms gives entropies from near 0 to near ln V
    hidden = (hidden.float() * torch.exp(torch.rand(B, N, 1, generator=g) * 5.0 - 3.0)).to(torch.bfloat16)
    w = (torch.randn(V, C, generator=g) * wstd).to(torch.bfloat16)
    b = (torch.randn(V, generator=g) * 0.5).to(torch.bfloat16) if bias else None
    return hidden, w, b


def _run(hidden, w, b, want_mean=True):
    nova = Hn.nova()
    B, N, C = hidden.shape
    V = w.shape[0]
    H = torch.full((B, N), float("nan"), dtype=torch.float32, device="cuda")
    mean = torch.empty(B, dtype=torch.float32, device="cuda") if want_mean else None
    ws = torch.empty(max(nova.head_entropy_workspace_bytes(N, B, V), 16), dtype=torch.uint8, device="cuda")
    nova.head_entropy(hidden.cuda(), w.cuda(), None if b is None else b.cuda(), H, ws, mean)
    torch.cuda.synchronize()
    return H.cpu().numpy(), None if mean is None else mean.cpu().numpy()


def _ok(got, ref):
    return np.all(np.abs(got - ref) <= 1e-4 * np.abs(ref) + 1e-5)


@pytest.mark.gpu
@pytest.mark.parametrize("B,N,C,V,bias", [
    (1, 1, 64, 32, True),            # one token, one narrow column tile
    (2, 37, 128, 500, True),         # ragged rows and a ragged last column tile
    (1, 300, 192, 4096, False),      # M <= 512: narrow staggered tiles
    (2, 700, 256, 1000, True),       # large tiles with ragged edges in both directions
    (3, 1024, 1024, 4096, True),     # several rounds of large tiles
])
def test_head_entropy_matches_oracle(B, N, C, V, bias):
    hidden, w, b = _case(B, N, C, V, seed=B * 1000 + N)
    got, mean = _run(hidden, w, b)
    ref = O.head_entropy(Hn.f64(hidden), Hn.f64(w), None if b is None else Hn.f64(b))
    assert np.isfinite(got).all()
    assert _ok(got, ref), float(np.max(np.abs(got - ref) / (1e-4 * np.abs(ref) + 1e-5)))
    if B * N >= 32:
        assert ref.min() < 0.5 * ref.max()      # the case really spans low and high entropies
    assert np.allclose(mean, ref.mean(axis=1), rtol=1e-4, atol=1e-5)


@pytest.mark.gpu
def test_head_entropy_cfg5_shape_sampled_rows():
    # the head of the largest workload: 2 x 4096 tokens, C = 2048, V = 4096; the oracle checks a sample of rows
    B, N, C, V = 2, 4096, 2048, 4096
    hidden, w, b = _case(B, N, C, V, seed=7, wstd=0.02)
    got, _ = _run(hidden, w, b, want_mean=False)
    assert np.isfinite(got).all() and got.min() >= 0.0 and got.max() <= np.log(V) * (1 + 1e-5)
    rows = np.random.default_rng(0).choice(N, size=96, replace=False)
    for bb in range(B):
        ref = O.head_entropy(Hn.f64(hidden[bb, rows]), Hn.f64(w), Hn.f64(b))
        assert _ok(got[bb, rows], ref)


@pytest.mark.gpu
def test_head_entropy_agrees_with_entropy_of_stored_logits():
    # the unfused route: logits rounded to bf16 and stored, then nova_entropy; both routes see the same head
    B, N, C, V = 2, 256, 256, 2048
    hidden, w, b = _case(B, N, C, V, seed=9)
    got, _ = _run(hidden, w, b, want_mean=False)
    logits = (hidden.float() @ w.float().T + b.float()).to(torch.bfloat16).cuda()
    H2 = torch.empty(B, N, dtype=torch.float32, device="cuda")
    Hn.nova().entropy(logits, H2)
    torch.cuda.synchronize()
    # bf16 storage perturbs each logit by up to 2^-9 relative: the entropies agree to about 1e-2
    assert np.allclose(got, H2.cpu().numpy(), rtol=2e-2, atol=2e-2)


@pytest.mark.gpu
def test_head_entropy_argument_errors():
    from paper_2602_01345_amd import NovaError
    nova = Hn.nova()
    h = torch.zeros(1, 4, 64, dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(32, 64, dtype=torch.bfloat16, device="cuda")
    H = torch.empty(1, 4, dtype=torch.float32, device="cuda")
    ws = torch.empty(nova.head_entropy_workspace_bytes(4, 1, 32), dtype=torch.uint8, device="cuda")
    with pytest.raises(NovaError):
        nova.head_entropy(h, w, None, H, ws[:16])                        # workspace too small
    with pytest.raises(NovaError):
        nova.head_entropy(h.float(), w.float(), None, H, ws)             # fp32 inputs are not supported
    h48 = torch.zeros(1, 4, 48, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(NovaError):
        nova.head_entropy(h48, w[:, :48].contiguous(), None, H, ws)      # C % 64 != 0


# ---------------------------------------------------------------------------------------------
# bitwise token heads
# ---------------------------------------------------------------------------------------------
@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("B,N,d", [(1, 1, 1), (2, 100, 32), (3, 257, 13), (2, 4096, 32), (1, 1000, 64)])
def test_entropy_bits_matches_oracle(dtype, B, N, d):
    g = torch.Generator().manual_seed(B * 31 + N + d)
    # per-token temperature: tokens from fully undecided to fully decided
    x = torch.randn(B, N, d, 2, generator=g) * torch.exp(torch.rand(B, N, 1, 1, generator=g) * 8.0 - 4.0)
    x = x.to(dtype)
    H = torch.empty(B, N, dtype=torch.float32, device="cuda")
    mean = torch.empty(B, dtype=torch.float32, device="cuda")
    Hn.nova().entropy_bits(x.cuda(), H, mean)
    torch.cuda.synchronize()
    ref = O.bitwise_entropy(Hn.f64(x))
    got = H.cpu().numpy()
    assert np.all(np.abs(got - ref) <= 1e-5 * np.abs(ref) + 1e-7 * d)
    assert np.allclose(mean.cpu().numpy(), ref.mean(axis=1), rtol=1e-5, atol=1e-6)


@pytest.mark.gpu
def test_entropy_bits_edge_values():
    x = torch.zeros(1, 6, 4, 2)
    x[0, 1, :, 1] = 300.0                       # certain bits
    x[0, 2, 0, 0] = float("inf")                # an infinite logit: that bit is certain
    x[0, 3, 1, 0] = float("-inf")
    x[0, 4, 2, 1] = float("nan")                # NaN propagates to the token
    x[0, 5, :, 0] = math.log(3.0)               # p = 1/4 on every bit
    H = torch.empty(1, 6, dtype=torch.float32, device="cuda")
    Hn.nova().entropy_bits(x.cuda(), H)
    got = H.cpu().numpy()[0]
    ln2 = math.log(2.0)
    assert got[0] == pytest.approx(4 * ln2, rel=1e-6)
    assert got[1] == 0.0
    assert got[2] == pytest.approx(3 * ln2, rel=1e-6) and got[3] == pytest.approx(3 * ln2, rel=1e-6)
    assert math.isnan(got[4])
    assert got[5] == pytest.approx(-4 * (0.25 * math.log(0.25) + 0.75 * math.log(0.75)), rel=1e-6)
    # unaligned base pointer (odd element offset): the scalar path
    y = torch.randn(2 * 7 * 2 + 1, dtype=torch.bfloat16, device="cuda")
    view = y[1:].view(1, 2, 7, 2)
    H2 = torch.empty(1, 2, dtype=torch.float32, device="cuda")
    Hn.nova().lib.nova_entropy_bits(Hn.nova().ctx, torch.cuda.current_stream().cuda_stream, view.data_ptr(), 1, 2, 1, 7,
                                    H2.data_ptr(), None)
    torch.cuda.synchronize()
    assert np.allclose(H2.cpu().numpy(), O.bitwise_entropy(Hn.f64(view)), rtol=1e-5)
