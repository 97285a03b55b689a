"""The library's host-side serialize(s_t) front end against the oracle, token for token (no GPU needed:
these entry points are host code), and - on a GPU - the chain state vectors -> ids -> frozen encoder -> heads
against the same chain through the oracles."""
import numpy as np
import pytest

from oracle import serialize_oracle as S
from paper_2604_24273_amd import synth


@pytest.fixture(scope="module")
def B():
    import os
    from paper_2604_24273_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2604_24273_amd import build
        build.build()
    binding.lib()
    return binding


def _special_values():
    vals = [0.0, -0.0, 0.25, 0.75, -0.25, 0.35, 0.05, -0.04, 0.049999997, 9.9, 9.94, 9.96, 10.0, -9.9, -12.0, 1e-30, -1e-30,
            1e-45, 3.4e38, -3.4e38, float("inf"), float("-inf"), float("nan"), 0.15, 2.5, 4.45, 9.85, 9.849999, 0.95]
    return np.asarray(vals, dtype=np.float32)


def test_text_and_ids_match_the_oracle(B):
    cases = [_special_values()] + [synth.normal(8, 800 + i, (n,), 3.0) for i, n in enumerate((1, 2, 17, 23, 27, 40, 300))]
    # every fp32 value on a fine grid around the rounding boundaries of one decade
    cases.append(np.arange(-1.2, 1.2, 0.0003, dtype=np.float32))
    for s in cases:
        s = np.ascontiguousarray(s, dtype=np.float32)
        text = B.brl_serialize_text(s)
        assert text == S.serialize_text(s)
        ids, cu = B.serialize_states(s.reshape(1, -1), 128256)
        assert list(ids) == S.serialize_ids(s)
        assert list(cu) == [0, len(s) + 2]
        assert B.brl_tokenize(text.encode("ascii")) == list(ids)


def test_neighbouring_floats_at_every_tie(B):
    # the two fp32 neighbours of every x.x5 boundary in [0, 9.9]: the library and the oracle agree on both sides
    pts = []
    for m in range(0, 99):
        t = np.float32((m + 0.5) / 10.0)
        pts += [np.nextafter(t, np.float32(-100)), t, np.nextafter(t, np.float32(100))]
    s = np.asarray(pts + [-p for p in pts], dtype=np.float32)
    ids, _ = B.serialize_states(s.reshape(1, -1), 457)
    assert list(ids) == S.serialize_ids(s)


def test_batch_layout_and_errors(B):
    states = np.ascontiguousarray(synth.normal(8, 820, (5, 19), 2.0))
    ids, cu = B.serialize_states(states, 1000)
    assert list(cu) == [21 * i for i in range(6)]
    for b in range(5):
        assert list(ids[cu[b]:cu[b + 1]]) == S.serialize_ids(states[b])
    with pytest.raises(B.BitrlError) as e:
        B.serialize_states(states, 456)                       # vocabulary too small for the ids used
    assert e.value.status == B.BRL_EINVAL


def test_tokenizer_on_free_text(B):
    for text in (b"", b"go north 1.5 then -0.5", b"state: 1.0state: -0.0 9.99 -9.9", bytes(range(256)), "café 3.5".encode("utf-8")):
        assert B.brl_tokenize(text) == S.tokenize(text)


@pytest.mark.gpu
def test_states_through_serialiser_encoder_and_heads():
    """17 - 27 dimensional states -> ids on the host -> encoder_forward_packed -> heads, against the oracles
    fed by the oracle's serialiser (cosine >= 0.999 per state, as for every encoder output)."""
    torch = pytest.importorskip("torch")
    from oracle import bitrl_oracle as O
    from paper_2604_24273_amd import binding as B
    from paper_2604_24273_amd import runtime as R
    B.lib()
    shape = synth.tiny_shape(n_layers=2, d=256, n_heads=4, n_kv_heads=2, head_dim=64, f=384, vocab=512, n_actions=6,
                             head_hidden=(32,))
    host = []
    enc = R.EncoderHandle(shape, seed=4, layer_sink=lambda l, w: host.append(w))
    head = R.HeadHandle(shape, seed=4)
    n_dims = 23
    states = np.ascontiguousarray(synth.normal(8, 830, (6, n_dims), 1.5))
    ids, cu = B.serialize_states(states, shape.vocab)
    h = enc.forward_packed(R.dev(ids), cu)
    logits, value = head.forward(h)
    torch.cuda.synchronize()
    T = O.TernaryLinear.from_fp32
    cfg = O.EncoderConfig(shape.n_layers, shape.d, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.f, shape.vocab,
                          shape.rope_theta)
    layers = [O.LayerWeights(w["attn_norm_g"], T(w["Wq"]), T(w["Wk"]), T(w["Wv"]), w["attn_subln_g"], T(w["Wo"]),
                             O.FFNWeights(w["ffn_norm_g"], T(w["W_gate"]), T(w["W_up"]), w["ffn_subln_g"], T(w["W_down"])))
              for w in host]
    emb, gfin = synth.embedding_bf16(4, shape), synth.final_norm_gain(4, shape)
    hg = h.cpu().numpy().astype(np.float64)
    for b in range(states.shape[0]):
        ref_ids = np.asarray(S.serialize_ids(states[b]), dtype=np.int32)[None, :]
        h_ref = O.encoder_forward(ref_ids, emb, layers, gfin, cfg)
        c = float(hg[b] @ h_ref[0] / np.linalg.norm(hg[b]) / np.linalg.norm(h_ref[0]))
        assert c >= 0.999, (b, c)
        l_ref, v_ref = O.policy_value_head(h_ref, O.MLP(*head.host["policy"], "tanh"), O.MLP(*head.host["value"], "tanh"))
        assert np.allclose(logits.cpu().numpy()[b], l_ref[0], rtol=1e-3, atol=1e-3 * float(np.abs(l_ref).max()))
