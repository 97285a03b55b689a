"""GPU parity of the attention stage by itself: attention_forward (the kernels encoder_forward runs on
the output of its q | k | v BitLinear) against the oracle's causal_gqa_attention, element by element.

Three kernels sit behind the entry point and every one is reached here in both layouts:
attention_f32_kernel (BRL_ATTN_F32), attn_pack_kernel + attention_frag_kernel (BRL_ATTN_MFMA) and
attention_short_kernel (BRL_ATTN_MFMA, states of at most 32 tokens).

Bound.  The oracle works in fp64 and rounds once.  The fp32 kernel accumulates dot products of
head_dim terms and the softmax sums in fp32; the matrix-core kernels carry every operand as an fp16
hi + lo pair (22 significant bits, the lo * lo term dropped) and accumulate in fp32.  With q, k, v of
unit scale a score then carries an absolute error of a few 1e-7 * sqrt(head_dim) before the
exponential, i.e. the probabilities a relative error of a few 1e-6, and the output (a convex
combination of v rows) the same relative to max|v|.  ATTN_REL below is that figure with a margin;
sharper softmaxes (inputs of three times the scale: nine times the score range) get nine times the
bound.
"""
import numpy as np
import pytest

from oracle import bitrl_oracle as O
from paper_2604_24273_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

ATTN_REL = 2e-6          # max |out - ref| / max |ref| per state, unit-scale inputs, either precision
                         # (largest seen over every case below: 5.3e-7 fp32, 4.1e-7 matrix cores; sharp case 3.5e-6)


def _mods():
    from paper_2604_24273_amd import binding as B
    from paper_2604_24273_amd import runtime as R
    B.lib()
    return B, R


def _run(B, R, qkv, lens, uniform_S, hq, hkv, dh, theta, prec, max_len=None):
    T = qkv.shape[0]
    nb = len(lens)
    out = torch.full((T, hq * dh), float("nan"), dtype=torch.float32, device="cuda")
    if uniform_S is not None:
        S, cu_dev, cu = uniform_S, None, None
    else:
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        cu_dev = R.dev(cu)
        S = max(lens) if max_len is None else max_len
    ws = R.Workspace(B.brl_attention_workspace_bytes(nb, S, hq, hkv, dh))
    B.attention_forward(R.dev(qkv), nb, S, cu_dev, cu, hq, hkv, dh, theta, prec, out, ws.buf)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def _oracle(qkv, lens, hq, hkv, dh, theta):
    outs, r0 = [], 0
    for n in lens:
        rows = qkv[r0:r0 + n]
        q = rows[:, :hq * dh].reshape(n, hq, dh)
        k = rows[:, hq * dh:(hq + hkv) * dh].reshape(n, hkv, dh)
        v = rows[:, (hq + hkv) * dh:].reshape(n, hkv, dh)
        outs.append(O.causal_gqa_attention(q, k, v, theta))
        r0 += n
    return outs


def _check(got, refs, lens, rel):
    r0, worst = 0, 0.0
    for n, ref in zip(lens, refs):
        g = got[r0:r0 + n].astype(np.float64)
        assert np.all(np.isfinite(g)), "rows of a state were not written"
        err = np.abs(g - ref.astype(np.float64)).max() / np.abs(ref).max()
        worst = max(worst, err)
        r0 += n
    print("   worst max|d|/max|ref| over %d states: %.3e (bound %.1e)" % (len(lens), worst, rel), flush=True)
    assert worst <= rel, "attention error %.3e above %.1e" % (worst, rel)


CASES = [
    # (head_dim, n_heads, n_kv_heads, state lengths, uniform layout?, rope theta)
    (128, 20, 5, [128, 128, 128], True, 500000.0),          # the 2B shape, one state = one 128-token block row
    (128, 4, 1, [1], True, 500000.0),
    (128, 4, 1, [32, 32], True, 500000.0),                    # one key block, uniform: the one-kernel path
    (128, 4, 1, [33, 33], True, 500000.0),                    # one token into the second key block
    (100, 4, 4, [512], True, 10000.0),                        # the 3B head: 100 components padded to 128, 16 key blocks
    (100, 2, 2, [33, 7, 70], False, 10000.0),
    (100, 2, 2, [19, 32, 5], False, 10000.0),                 # short states, head_dim 100
    (16, 8, 1, [9, 40, 64], False, 10000.0),                  # eight query heads per key/value head
    (16, 8, 1, [9, 31], False, 10000.0),
    (32, 8, 8, [31, 17, 32], False, 10000.0),
    (64, 4, 2, [15, 40, 1, 32, 33, 27, 64, 31], False, 10000.0),
    (64, 8, 1, [15, 27, 1, 32, 8], False, 10000.0),           # 8:1 grouping, all short
    (128, 8, 2, [129, 2, 96, 18, 40], False, 500000.0),
]


@pytest.mark.parametrize("prec", ["f32", "mfma"])
@pytest.mark.parametrize("dh,hq,hkv,lens,uniform,theta", CASES)
def test_attention_stage_against_oracle(dh, hq, hkv, lens, uniform, theta, prec):
    B, R = _mods()
    print("attention_forward", dh, hq, hkv, lens, uniform, prec, flush=True)
    T = int(np.sum(lens))
    qkv = synth.normal(7, 600 + dh + len(lens), (T, (hq + 2 * hkv) * dh))
    p = B.BRL_ATTN_F32 if prec == "f32" else B.BRL_ATTN_MFMA
    got = _run(B, R, qkv, lens, lens[0] if uniform else None, hq, hkv, dh, theta, p)
    _check(got, _oracle(qkv, lens, hq, hkv, dh, theta), lens, ATTN_REL)
    if not uniform:
        # a larger bound on the lengths changes nothing, bit for bit
        again = _run(B, R, qkv, lens, None, hq, hkv, dh, theta, p, max_len=max(lens) + 37)
        assert np.array_equal(got, again)


@pytest.mark.parametrize("prec", ["f32", "mfma"])
def test_attention_sharp_softmax(prec):
    """Inputs of three times the scale: scores range over about +-30, the running-maximum form must hold."""
    B, R = _mods()
    dh, hq, hkv, lens = 128, 4, 2, [96, 40, 23]
    qkv = synth.normal(7, 650, (int(np.sum(lens)), (hq + 2 * hkv) * dh), 3.0)
    p = B.BRL_ATTN_F32 if prec == "f32" else B.BRL_ATTN_MFMA
    got = _run(B, R, qkv, lens, None, hq, hkv, dh, 500000.0, p)
    _check(got, _oracle(qkv, lens, hq, hkv, dh, 500000.0), lens, 9 * ATTN_REL)


def test_attention_many_short_states_take_the_two_kernel_path():
    """More than 1024 (state, key/value head) workgroups of short states: the pack + fragment kernels run
    with a single key block.  The same rows through the one-kernel path (few states per call) must agree with
    the oracle to the same bound; both are compared with it."""
    B, R = _mods()
    dh, hq, hkv = 64, 4, 4
    lens = [int(n) for n in synth.state_lengths(7, 660, 300, 1, 32)]       # 300 x 4 = 1200 workgroups
    qkv = synth.normal(7, 661, (int(np.sum(lens)), (hq + 2 * hkv) * dh))
    refs = _oracle(qkv, lens, hq, hkv, dh, 10000.0)
    got = _run(B, R, qkv, lens, None, hq, hkv, dh, 10000.0, B.BRL_ATTN_MFMA)
    _check(got, refs, lens, ATTN_REL)
    few = 40
    t_few = int(np.sum(lens[:few]))
    got_few = _run(B, R, qkv[:t_few], lens[:few], None, hq, hkv, dh, 10000.0, B.BRL_ATTN_MFMA)
    _check(got_few, refs[:few], lens[:few], ATTN_REL)
    # same block arithmetic in both kernels: identical bits
    assert np.array_equal(got[:t_few], got_few)


def test_attention_is_causal_and_state_local():
    """Changing the tokens behind a position, or another state, leaves that position's output unchanged bit
    for bit (a property that holds at any size; both precisions)."""
    B, R = _mods()
    dh, hq, hkv, lens = 128, 4, 1, [70, 45]
    T = int(np.sum(lens))
    qkv = synth.normal(7, 670, (T, (hq + 2 * hkv) * dh))
    other = qkv.copy()
    other[50:70] = synth.normal(7, 671, (20, qkv.shape[1]))     # the tail of state 0
    other[70:] = synth.normal(7, 672, (45, qkv.shape[1]))       # all of state 1
    for p in (B.BRL_ATTN_F32, B.BRL_ATTN_MFMA):
        a = _run(B, R, qkv, lens, None, hq, hkv, dh, 500000.0, p)
        b = _run(B, R, other, lens, None, hq, hkv, dh, 500000.0, p)
        assert np.array_equal(a[:50], b[:50])
        assert not np.array_equal(a[50:70], b[50:70])


def test_attention_argument_checks():
    B, R = _mods()
    qkv = R.dev(synth.normal(7, 680, (8, 3 * 64)))
    out = torch.empty((8, 64), dtype=torch.float32, device="cuda")
    ws = R.Workspace(B.brl_attention_workspace_bytes(1, 8, 1, 1, 64))
    with pytest.raises(B.BitrlError) as e:
        B.attention_forward(qkv, 1, 8, None, None, 1, 1, 48, 10000.0, B.BRL_ATTN_MFMA, out, ws.buf)
    assert e.value.status == B.BRL_EINVAL
    with pytest.raises(B.BitrlError) as e:
        B.attention_forward(qkv, 1, 8, None, None, 3, 2, 64, 10000.0, B.BRL_ATTN_MFMA, out, ws.buf)
    assert e.value.status == B.BRL_EINVAL
    cu = np.asarray([0, 9], dtype=np.int32)                   # longer than the bound S = 8
    with pytest.raises(B.BitrlError) as e:
        B.attention_forward(qkv, 1, 8, R.dev(cu), cu, 1, 1, 64, 10000.0, B.BRL_ATTN_MFMA, out, ws.buf)
    assert e.value.status == B.BRL_EINVAL
    small = R.Workspace(64)
    with pytest.raises(B.BitrlError) as e:
        B.attention_forward(qkv, 1, 8, None, None, 1, 1, 64, 10000.0, B.BRL_ATTN_MFMA, out, small.buf)
    assert e.value.status == B.BRL_ENOSPC
