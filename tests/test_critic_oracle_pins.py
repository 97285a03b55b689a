"""Pins for oracle/critic_oracle.py: the int8-weight BitLinear and the ensemble critic.

Nothing here comes from the GPU path.  Each check ties the oracle to something other than
itself: hand-worked cases (tests/golden), exact integer special cases, error bounds that
follow from the definition, symmetries, pure-Python brute force on tiny inputs, and special
cases that reduce to a plain linear map."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import bitrl_oracle as O
from oracle import critic_oracle as C

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
F32 = np.float32


def _rows(txt):
    return [[float(v) for v in r.split()] for r in txt.split(";")]


def _hand_cases():
    out = []
    with open(os.path.join(GOLDEN, "int8_weight_hand_cases.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w, c, s = [p.strip() for p in line.split("|")]
            num, den = s.split("/")
            out.append((np.array(_rows(w), dtype=F32), np.array(_rows(c), dtype=np.int64), float(num) / float(den)))
    return out


def test_hand_worked_cases():
    cases = _hand_cases()
    assert len(cases) == 5
    for W, codes, scale in cases:
        got, s = C.int8_quantize(W, 1e-5)
        assert got.dtype == np.int8 and np.array_equal(got.astype(np.int64), codes)
        assert abs(float(s) - scale) <= 1e-7 * scale


def test_integer_matrix_with_max_127_is_reproduced_exactly():
    rng = np.random.default_rng(1)
    W = rng.integers(-127, 128, size=(9, 33)).astype(F32)
    W[4, 7] = 127.0
    codes, s = C.int8_quantize(W)
    assert np.array_equal(codes.astype(F32), W) and s == F32(1.0)
    # ... and then the whole layer is an exact integer product times the token scale
    x = rng.integers(-127, 128, size=(5, 33)).astype(F32)
    x[:, 0] = 127.0
    y = C.int8_bitlinear_forward(x, codes, s)
    want = x.astype(np.int64) @ W.astype(np.int64).T        # a_t = 127 -> a_t / 127 = 1
    assert np.array_equal(y.astype(np.float64), want.astype(np.float64))


def test_reconstruction_error_is_half_a_step():
    rng = np.random.default_rng(2)
    W = (rng.standard_normal((40, 70)) * 0.02).astype(F32)
    codes, s = C.int8_quantize(W)
    a = np.abs(W).max()
    assert codes.min() >= -127 and codes.max() <= 127
    assert np.abs(codes[np.unravel_index(np.abs(W).argmax(), W.shape)]) == 127
    err = np.abs(codes.astype(np.float64) * float(s) - W.astype(np.float64)).max()
    assert err <= float(a) / 254.0 * (1 + 1e-5)
    # a dropped rounding (truncation) or a 128-level grid would break the bound or the next line
    assert abs(float(s) * 127.0 - float(a)) <= 1e-7 * float(a)


def test_power_of_two_scaling_and_sign_symmetry():
    rng = np.random.default_rng(3)
    W = rng.standard_normal((16, 24)).astype(F32)
    c0, s0 = C.int8_quantize(W)
    for k in (-6, 3, 10):
        c, s = C.int8_quantize(W * F32(2.0 ** k))
        assert np.array_equal(c, c0) and s == F32(float(s0) * 2.0 ** k)
    cn, sn = C.int8_quantize(-W)
    assert np.array_equal(cn, -c0) and sn == s0
    # one scale for the whole matrix, not one per row: permuting rows permutes codes
    perm = rng.permutation(16)
    cp, sp = C.int8_quantize(W[perm])
    assert np.array_equal(cp, c0[perm]) and sp == s0


def test_brute_force_tiny_layer():
    rng = np.random.default_rng(4)
    W = rng.standard_normal((3, 5)).astype(F32)
    x = rng.standard_normal((2, 5)).astype(F32)
    codes, s = C.int8_quantize(W)
    taps = {}
    y = C.int8_bitlinear_forward(x, codes, s, taps=taps)
    for t in range(2):
        a = max(max(abs(float(v)) for v in x[t]), 1e-5)
        sc = F32(F32(127) / F32(a))
        q = [int(np.clip(np.rint(F32(v) * sc), -127, 127)) for v in x[t]]
        assert q == taps["xq"][t].tolist()
        for n in range(3):
            acc = sum(q[k] * int(codes[n, k]) for k in range(5))
            assert acc == int(taps["acc"][t, n])
            want = F32(F32(F32(acc) * F32(F32(a) / F32(127))) * s)
            assert y[t, n] == want


def test_layer_is_close_to_the_unquantised_product():
    rng = np.random.default_rng(5)
    K = 256
    W = (rng.standard_normal((32, K)) * 0.05).astype(F32)
    x = rng.standard_normal((8, K)).astype(F32)
    codes, s = C.int8_quantize(W)
    y = C.int8_bitlinear_forward(x, codes, s).astype(np.float64)
    ref = x.astype(np.float64) @ W.astype(np.float64).T
    a_w = float(np.abs(W).max())
    a_x = np.abs(x).max(axis=1).astype(np.float64)
    # |dx| <= a_x/254, |dW| <= a_w/254 per element: deterministic bound on the product error
    l1x = np.abs(x).sum(axis=1).astype(np.float64)
    l1w = np.abs(W).sum(axis=1).astype(np.float64)
    bound = (l1x[:, None] * a_w / 254 + a_x[:, None] / 254 * l1w[None, :] + K * a_x[:, None] * a_w / 254 ** 2) * 1.001
    assert np.all(np.abs(y - ref) <= bound)
    # and in practice far inside it: a transposed operand or a wrong scale gives O(1) relative error
    assert np.abs(y - ref).max() <= 0.02 * np.abs(ref).max()
    # residual is added after the rescale
    r = rng.standard_normal((8, 32)).astype(F32)
    y2 = C.int8_bitlinear_forward(x, codes, s, residual=r)
    assert np.array_equal(y2, (C.int8_bitlinear_forward(x, codes, s) + r).astype(F32))


def test_int8_linear_drops_into_the_block_definitions():
    rng = np.random.default_rng(6)
    d, f, M = 32, 48, 6
    x = rng.standard_normal((M, d)).astype(F32)
    mk = lambda n, k: C.Int8Linear.from_fp32((rng.standard_normal((n, k)) * 0.1).astype(F32))
    w = O.FFNWeights(np.ones(d, F32), mk(f, d), mk(f, d), np.ones(f, F32), mk(d, f))
    y = O.ffn_block_forward(x, w)
    # the same block written out with the int8 layer function
    n = O.rmsnorm(x, w.norm_g)
    G = C.int8_bitlinear_forward(n, w.gate.codes, w.gate.beta)
    U = C.int8_bitlinear_forward(n, w.up.codes, w.up.beta)
    m = O.rmsnorm(O.squared_relu_glu(G, U), w.subln_g)
    assert np.array_equal(y, C.int8_bitlinear_forward(m, w.down.codes, w.down.beta, residual=x))


def _mlp(rng, dims, act="tanh"):
    ws = [(rng.standard_normal((dims[i + 1], dims[i])) / np.sqrt(dims[i])).astype(F32) for i in range(len(dims) - 1)]
    bs = [(rng.standard_normal(dims[i + 1]) * 0.1).astype(F32) for i in range(len(dims) - 1)]
    return O.MLP(ws, bs, act)


def test_ensemble_of_identical_members_is_the_member():
    rng = np.random.default_rng(7)
    m = _mlp(rng, [20, 8, 1])
    h = rng.standard_normal((9, 20)).astype(F32)
    mean, each = C.value_ensemble(h, [m, m, m])
    v = O.mlp_forward(h, m)[:, 0]
    assert each.shape == (3, 9) and np.array_equal(each[0], v) and np.array_equal(each[2], v)
    assert np.array_equal(mean, v)          # (3 v) / 3 in fp64 rounds back to the fp32 v
    one, e1 = C.value_ensemble(h, [m])
    assert np.array_equal(one, v) and e1.shape == (1, 9)


def test_ensemble_mean_by_exact_rational_arithmetic():
    rng = np.random.default_rng(8)
    members = [_mlp(rng, [12, 6, 1], "relu") for _ in range(5)]
    h = rng.standard_normal((4, 12)).astype(F32)
    mean, each = C.value_ensemble(h, members)
    for i, m in enumerate(members):
        assert np.array_equal(each[i], O.mlp_forward(h, m)[:, 0])
    for b in range(4):
        exact = sum(Fraction(float(each[i, b])) for i in range(5)) / 5
        assert abs(Fraction(float(mean[b])) - exact) <= abs(exact) * Fraction(1, 2 ** 23) + Fraction(1, 2 ** 120)
    # order of members does not matter beyond rounding; a sum instead of a mean would be 5x off
    mean_r, _ = C.value_ensemble(h, members[::-1])
    assert np.allclose(mean_r, mean, rtol=2e-7, atol=1e-12)


def test_linear_members_average_like_their_parameters():
    rng = np.random.default_rng(9)
    members = [_mlp(rng, [16, 1]) for _ in range(3)]
    h = rng.standard_normal((7, 16)).astype(F32)
    mean, _ = C.value_ensemble(h, members)
    Wm = np.mean([m.weights[0].astype(np.float64) for m in members], axis=0)
    bm = np.mean([m.biases[0].astype(np.float64) for m in members], axis=0)
    ref = h.astype(np.float64) @ Wm.T + bm
    assert np.abs(mean - ref[:, 0]).max() <= 5e-7 * np.abs(ref).max() + 1e-7


def test_int4_grid_hand_case_and_bounds():
    # max 1 -> s = 7: 0.5 -> 3.5 -> 4 (even), 0.25 -> 1.75 -> 2, -0.75 -> -5.25 -> -5, 0.0714 -> 0.4998 -> 0
    W = np.array([[1.0, -0.5, 0.25, 0.0], [0.5, -0.75, -1.0, 0.0714]], dtype=F32)
    codes, s = C.int8_quantize(W, qmax=7)
    assert codes.tolist() == [[7, -4, 2, 0], [4, -5, -7, 0]]
    assert abs(float(s) - 1.0 / 7.0) <= 1e-8
    rng = np.random.default_rng(11)
    W = (rng.standard_normal((30, 50)) * 0.02).astype(F32)
    c7, s7 = C.int8_quantize(W, qmax=7)
    assert c7.min() >= -7 and c7.max() <= 7 and np.abs(c7).max() == 7
    a = float(np.abs(W).max())
    assert np.abs(c7.astype(np.float64) * float(s7) - W).max() <= a / 14.0 * (1 + 1e-5)
    # an integer matrix with max 7 is reproduced exactly, and the coarser grid is coarser
    Wi = rng.integers(-7, 8, size=(6, 9)).astype(F32); Wi[0, 0] = 7
    ci, si = C.int8_quantize(Wi, qmax=7)
    assert np.array_equal(ci.astype(F32), Wi) and si == F32(1.0)
    c127, s127 = C.int8_quantize(W)
    e7 = np.abs(c7.astype(np.float64) * float(s7) - W).mean()
    e127 = np.abs(c127.astype(np.float64) * float(s127) - W).mean()
    assert e7 > 10 * e127
    with pytest.raises(ValueError):
        C.int8_quantize(W, qmax=0)
    with pytest.raises(ValueError):
        C.int8_quantize(W, qmax=128)


def test_errors():
    with pytest.raises(ValueError):
        C.value_ensemble(np.zeros((2, 4), F32), [])
    with pytest.raises(ValueError):
        C.int8_quantize(np.array([[np.inf, 1.0]], dtype=F32))
    rng = np.random.default_rng(10)
    with pytest.raises(ValueError):
        C.value_ensemble(np.zeros((2, 4), F32), [_mlp(rng, [4, 2])])
