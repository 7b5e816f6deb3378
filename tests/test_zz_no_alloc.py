"""The allocation-free entry point (nova_head_entropy_static: per-tile entropy partials in the library's static
device scratch instead of a caller's workspace) against the existing entry point it is a variant of
(nova_head_entropy), through the C ABI: two calls in a row, the second with a smaller input that leaves stale
partials of the first call behind it in the scratch.  Same kernels, same order of operations: the results must
be the same bits; they are also held to the oracle at nova_head_entropy's tolerance."""
import ctypes as C

import numpy as np
import pytest
import torch

import harness as Hn
from oracle import nova_oracle as O

pytestmark = pytest.mark.gpu


def _case(B, N, Cw, V, seed):
    g = torch.Generator().manual_seed(seed)
    hidden = torch.randn(B, N, Cw, generator=g)
    hidden = (hidden * torch.exp(torch.rand(B, N, 1, generator=g) * 5.0 - 3.0)).to(torch.bfloat16)
    w = (torch.randn(V, Cw, generator=g) * 0.05).to(torch.bfloat16)
    b = (torch.randn(V, generator=g) * 0.5).to(torch.bfloat16)
    return hidden, w, b


def _both(nova, hidden, w, b):
    """(static entry point, workspace entry point) results of one input, both through the raw C ABI."""
    lib = nova.lib
    B, N, Cw = hidden.shape
    V = w.shape[0]
    hd, wd, bd = hidden.cuda(), w.cuda(), b.cuda()
    out = []
    for static in (True, False):
        H = torch.full((B, N), float("nan"), dtype=torch.float32, device="cuda")
        mean = torch.full((B,), float("nan"), dtype=torch.float32, device="cuda")
        if static:
            rc = lib.nova_head_entropy_static(nova.ctx, None, hd.data_ptr(), wd.data_ptr(), bd.data_ptr(), 1, N, B,
                                              Cw, V, H.data_ptr(), mean.data_ptr())
        else:
            need = lib.nova_head_entropy_workspace_bytes(N, B, V)
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            rc = lib.nova_head_entropy(nova.ctx, None, hd.data_ptr(), wd.data_ptr(), bd.data_ptr(), 1, N, B, Cw, V,
                                       H.data_ptr(), mean.data_ptr(), ws.data_ptr(), C.c_size_t(need))
        assert rc == 0, rc
        torch.cuda.synchronize()
        out.append((H.cpu().numpy(), mean.cpu().numpy()))
    return out


def test_static_scratch_entry_point_matches_the_workspace_one_on_two_calls_in_a_row():
    nova = Hn.nova()
    # first call: several rounds of large tiles; second call: fewer rows, fewer column tiles, ragged edges
    for B, N, Cw, V, seed in ((3, 1024, 512, 4096, 1), (2, 37, 128, 500, 2)):
        print(f"no-alloc head entropy B={B} N={N} C={Cw} V={V}", flush=True)
        hidden, w, b = _case(B, N, Cw, V, seed)
        (Hs, ms), (Hw, mw) = _both(nova, hidden, w, b)
        assert np.isfinite(Hs).all() and np.isfinite(ms).all()
        assert np.array_equal(Hs, Hw) and np.array_equal(ms, mw)
        ref = O.head_entropy(Hn.f64(hidden), Hn.f64(w), Hn.f64(b))
        assert np.all(np.abs(Hs - ref) <= 1e-4 * np.abs(ref) + 1e-5)
        assert np.allclose(ms, ref.mean(axis=1), rtol=1e-4, atol=1e-5)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    nova = Hn.nova()
    hidden, w, b = _case(1, 8, 64, 64, 3)
    hd, wd, bd = hidden.cuda(), w.cuda(), b.cuda()
    H = torch.zeros(8, dtype=torch.float32, device="cuda")
    # 2^20 rows of V = 4096 would need 16 partial tiles x 16 MiB: refused on the host, nothing is launched
    rc = nova.lib.nova_head_entropy_static(nova.ctx, None, hd.data_ptr(), wd.data_ptr(), bd.data_ptr(), 1, 1 << 20, 1,
                                           64, 4096, H.data_ptr(), None)
    assert rc == -5
    assert b"static scratch" in nova.lib.nova_strerror(rc)
    torch.cuda.synchronize()
    assert float(H.abs().sum()) == 0.0
