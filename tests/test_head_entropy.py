"""Entropy straight from a linear head (Sec. 4, "Entropy Computation Overhead") against the oracle's
composition entropy(hidden W^T + b).  Tolerance: the logits are fp32 sums of exact bf16 products
(K <= 2304 terms), so |dH| <= 1e-4 |H| + 1e-5 covers accumulation order and the fp32 softmax sums."""
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
