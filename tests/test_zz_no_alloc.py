"""bitlinear_forward_static (the entry point that allocates nothing: its scratch is an array built into the
library) against bitlinear_forward, bit for bit, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest

from paper_2604_24273_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _mods():
    from paper_2604_24273_amd import binding as B
    from paper_2604_24273_amd import runtime as R
    B.lib()
    return B, R


def _both(B, R, pl, x, M, N, K, residual):
    outs = []
    for static in (False, True):
        y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        xq = torch.zeros((M, K), dtype=torch.int8, device="cuda")
        am = torch.zeros((M,), dtype=torch.float32, device="cuda")
        acc = torch.zeros((M, N), dtype=torch.int32, device="cuda")
        for taps in (True, False):          # with taps (per-element epilogue) and without (16-byte epilogue)
            t = (xq, am, acc) if taps else (None, None, None)
            if static:
                B.bitlinear_forward_static(pl.packed, pl.beta, N, K, x, M, 1e-5, y, residual, *t)
            else:
                ws = R.Workspace(B.brl_bitlinear_workspace_bytes(M, N, K))
                B.bitlinear_forward(pl.packed, pl.beta, N, K, x, M, 1e-5, y, residual, *t, ws.buf)
            torch.cuda.synchronize()
            outs.append((y.clone(), xq.clone(), am.clone(), acc.clone()))
    half = len(outs) // 2
    for a, b in zip(outs[:half], outs[half:]):
        for ta, tb in zip(a, b):
            assert torch.equal(ta, tb)
    assert bool(torch.isfinite(outs[-1][0]).all())


def test_static_scratch_entry_point_two_calls_second_smaller():
    B, R = _mods()
    # first call: 300 tokens x 6912 features (a product bitlinear_forward cuts along k; here it runs uncut)
    N1, K1, M1 = 2560, 6912, 300
    pl1 = R.quantize_linear(synth.normal(11, 1, (N1, K1), 0.02))
    x1 = R.dev(synth.normal(11, 2, (M1, K1)))
    res1 = R.dev(synth.normal(11, 3, (M1, N1)))
    _both(B, R, pl1, x1, M1, N1, K1, res1)
    # second call, smaller in both dimensions, ragged: 45 tokens x 200 features; the array still holds the first call's bytes
    N2, K2, M2 = 70, 200, 45
    pl2 = R.quantize_linear(synth.normal(11, 4, (N2, K2), 0.02))
    x2 = R.dev(synth.normal(11, 5, (M2, K2)))
    _both(B, R, pl2, x2, M2, N2, K2, None)
    # a bf16 input and the 1..4 token path (no scratch)
    x3 = R.bf16_from_bits(synth.to_bf16_bits(synth.normal(11, 6, (3, K1))))
    _both(B, R, pl1, x3, 3, N1, K1, None)
    # a many-token product (the 128 x 256 tile kernel) right after the small ones
    M4 = 2048
    x4 = R.dev(synth.normal(11, 7, (M4, K1)))
    _both(B, R, pl1, x4, M4, N1, K1, None)


def test_static_scratch_rejects_what_does_not_fit():
    B, R = _mods()
    N, K = 64, 6912
    pl = R.quantize_linear(synth.normal(11, 8, (N, K), 0.02))
    M = 2432                                     # 2432 x 6912 bytes > 16 MiB
    x = torch.zeros((M, K), dtype=torch.float32, device="cuda")
    y = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    with pytest.raises(B.BitrlError) as e:
        B.bitlinear_forward_static(pl.packed, pl.beta, N, K, x, M, 1e-5, y, None, None, None, None)
    assert e.value.status == B.BRL_ENOSPC
    assert "scratch" in str(e.value)
