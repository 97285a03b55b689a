"""GPU parity at the full benchmark sizes, on sampled states the oracle can afford.

States are independent (frozen, stateless encoder), so a sampled state of the
full batch has exactly one correct answer, which the oracle computes alone.
The GPU side runs the whole batch in the launch configuration bench.py times.
"""
import numpy as np
import pytest

from oracle import bitrl_oracle as O
from paper_2604_24273_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _cos(a, b):
    a = np.asarray(a, np.float64).ravel(); b = np.asarray(b, np.float64).ravel()
    return float(a @ b / (np.linalg.norm(a) * np.linalg.norm(b)))


def _oracle_layers(host):
    T = O.TernaryLinear.from_fp32
    return [O.LayerWeights(w["attn_norm_g"], T(w["Wq"]), T(w["Wk"]), T(w["Wv"]), w["attn_subln_g"], T(w["Wo"]),
                           O.FFNWeights(w["ffn_norm_g"], T(w["W_gate"]), T(w["W_up"]), w["ffn_subln_g"], T(w["W_down"])))
            for w in host]


def _oracle_layers_int8(host):
    from oracle import critic_oracle as C
    T = C.Int8Linear.from_fp32
    return [O.LayerWeights(w["attn_norm_g"], T(w["Wq"]), T(w["Wk"]), T(w["Wv"]), w["attn_subln_g"], T(w["Wo"]),
                           O.FFNWeights(w["ffn_norm_g"], T(w["W_gate"]), T(w["W_up"]), w["ffn_subln_g"], T(w["W_down"])))
            for w in host]


def _build(shape, seed, int8_twin=False):
    from paper_2604_24273_amd import binding as B
    from paper_2604_24273_amd import runtime as R
    B.lib()
    layers, layers8 = [], []

    def sink(l, w):
        # quantise the oracle's copy right away so the fp32 masters can be dropped
        layers.extend(_oracle_layers([w]))
        if int8_twin:
            layers8.extend(_oracle_layers_int8([w]))

    enc = R.EncoderHandle(shape, seed=seed, layer_sink=sink, int8_twin=int8_twin)
    cfg = O.EncoderConfig(shape.n_layers, shape.d, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.f,
                          shape.vocab, shape.rope_theta)
    if int8_twin:
        return B, R, enc, cfg, layers, layers8
    return B, R, enc, cfg, layers


@pytest.mark.timeout(1500)
def test_encoder_2b_shape_full_batch_sampled_states():
    """30 layers, hidden 2560, 20/5 heads, FFN 6912, vocab 128256; 64 states x 128 tokens; heads 2560->256->18 / 1."""
    shape = synth.SHAPE_2B
    print("encoder 2B shape: building", flush=True)
    B, R, enc, cfg, layers, layers8 = _build(shape, 0, int8_twin=True)
    head = R.HeadHandle(shape, seed=0)
    ids = synth.token_ids(0, 500, (64, 128), shape.vocab)
    print("encoder 2B shape: GPU forward", flush=True)
    h = enc.forward(R.dev(ids))
    logits, value = head.forward(h)
    hg = h.cpu().numpy()
    assert np.all(np.isfinite(hg))
    emb = synth.embedding_bf16(0, shape)
    gfin = synth.final_norm_gain(0, shape)
    sample = [0, 37]
    print("encoder 2B shape: oracle on states", sample, flush=True)
    h_ref = O.encoder_forward(ids[sample], emb, layers, gfin, cfg)
    l_ref, v_ref = O.policy_value_head(h_ref, O.MLP(*head.host["policy"], "tanh"), O.MLP(*head.host["value"], "tanh"))
    for j, b in enumerate(sample):
        c = _cos(hg[b], h_ref[j])
        print("state %d: cosine %.7f, max rel err %.3e" % (b, c, np.abs(hg[b] - h_ref[j]).max() / np.abs(h_ref[j]).max()), flush=True)
        assert c >= 0.999
        assert _cos(logits.cpu().numpy()[b], l_ref[j]) >= 0.999
        assert abs(float(value.cpu().numpy()[b]) - float(v_ref[j])) <= 0.05 * max(1.0, abs(float(v_ref[j])))
    # batch invariance and run-to-run identity at the benchmark launch configuration
    assert torch.equal(h, enc.forward(R.dev(ids)))
    assert torch.equal(h[37:38], enc.forward(R.dev(ids[37:38])))
    # variable-length states: the first 20 tokens of state 37, padded to 128
    lengths = np.full(64, 128, np.int32); lengths[37] = 20
    hl = enc.forward(R.dev(ids), R.dev(lengths)).cpu().numpy()
    h20 = O.encoder_forward(ids[37:38, :20], emb, layers, gfin, cfg)
    assert _cos(hl[37], h20[0]) >= 0.999
    assert np.array_equal(hl[0], hg[0])
    # the packed entry point in the configuration `bench.py --workload rl-states-2b` times:
    # 1024 states of 15-40 tokens stored back to back; state 37 is again those 20 tokens
    lens = synth.state_lengths(0, 501, 1024, 15, 40)
    lens[37] = 20
    wide = synth.token_ids(0, 500, (1024, 40), shape.vocab)
    wide[37, :20] = ids[37, :20]
    flat = np.concatenate([wide[i, :n] for i, n in enumerate(lens)]).astype(np.int32)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    print("encoder 2B shape: packed batch of 1024 states, %d tokens" % cu[-1], flush=True)
    hp = enc.forward_packed(R.dev(flat), cu, max_len=40).cpu().numpy()
    assert np.all(np.isfinite(hp))
    assert _cos(hp[37], h20[0]) >= 0.999
    assert np.array_equal(hp[37], hl[37])      # padded or packed, among 64 or among 1024 states: the same bits
    # one short state per call (the deployment shape): per-token quantisation, k-split GEMMs, one-kernel attention
    print("encoder 2B shape: one 20-token state", flush=True)
    h1 = enc.forward_packed(R.dev(ids[37, :20].astype(np.int32)), np.asarray([0, 20], np.int32)).cpu().numpy()
    assert _cos(h1[0], h20[0]) >= 0.999
    assert np.abs(h1[0] - hl[37]).max() <= 1e-3 * np.abs(hl[37]).max()
    # the int8-weight encoder of the same master weights (critic backbone), same batch, sampled state
    print("encoder 2B shape: int8-weight twin", flush=True)
    h8 = enc.int8_twin.forward(R.dev(ids)).cpu().numpy()
    assert np.all(np.isfinite(h8))
    h8_ref = O.encoder_forward(ids[37:38], emb, layers8, gfin, cfg)
    c8 = _cos(h8[37], h8_ref[0])
    print("int8 weights, state 37: cosine %.7f" % c8, flush=True)
    assert c8 >= 0.999


@pytest.mark.timeout(1500)
def test_encoder_3b_shape_prefill_microbatch_sampled_state():
    """26 layers, hidden 3200, 32 heads of 100, FFN 8640, vocab 32000; 512-token states.  The full
    workload is 1024 states in micro-batches of 64; the GPU runs one whole micro-batch (64 states x 512
    tokens = 32 768 token rows: the launch configuration bench.py times), the oracle affords one
    sampled state of it."""
    shape = synth.SHAPE_3B
    print("encoder 3B shape: building", flush=True)
    B, R, enc, cfg, layers = _build(shape, 0)
    ids = synth.token_ids(0, 500, (64, 512), shape.vocab)
    print("encoder 3B shape: GPU forward, 64 states x 512 tokens", flush=True)
    h = enc.forward(R.dev(ids))
    hg = h.cpu().numpy()
    assert np.all(np.isfinite(hg))
    emb = synth.embedding_bf16(0, shape)
    gfin = synth.final_norm_gain(0, shape)
    sample = 41
    print("encoder 3B shape: oracle on state", sample, flush=True)
    h_ref = O.encoder_forward(ids[sample:sample + 1], emb, layers, gfin, cfg)
    c = _cos(hg[sample], h_ref[0])
    print("state %d: cosine %.7f, max rel err %.3e" % (sample, c, np.abs(hg[sample] - h_ref[0]).max() / np.abs(h_ref[0]).max()),
          flush=True)
    assert c >= 0.999
    # batch invariance: the state alone (a 512-token launch configuration) gives the same bits
    assert torch.equal(h[sample:sample + 1], enc.forward(R.dev(ids[sample:sample + 1])))
    assert torch.equal(h, enc.forward(R.dev(ids)))


def test_encoder_micro_batching_is_invisible():
    """More tokens than one micro-batch holds: results equal those of the states run in small groups."""
    from paper_2604_24273_amd import runtime as R
    shape = synth.tiny_shape(n_layers=1, d=64, n_heads=2, n_kv_heads=1, head_dim=32, f=128, vocab=200)
    host = []
    enc = R.EncoderHandle(shape, seed=2, layer_sink=lambda l, w: host.append(w))
    ids = synth.token_ids(2, 500, (600, 64), shape.vocab)          # 38400 tokens > 32768
    lengths = synth.state_lengths(2, 501, 600, 1, 64)
    h = enc.forward(R.dev(ids), R.dev(lengths))
    for lo, hi in ((0, 7), (505, 520), (590, 600)):
        part = enc.forward(R.dev(ids[lo:hi]), R.dev(lengths[lo:hi]))
        assert torch.equal(h[lo:hi], part)
    cfg = O.EncoderConfig(shape.n_layers, shape.d, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.f,
                          shape.vocab, shape.rope_theta)
    sample = [3, 511, 512, 599]
    h_ref = O.encoder_forward(ids[sample], synth.embedding_bf16(2, shape), _oracle_layers(host),
                              synth.final_norm_gain(2, shape), cfg, lengths=lengths[sample])
    for j, b in enumerate(sample):
        assert _cos(h.cpu().numpy()[b], h_ref[j]) >= 0.999


@pytest.mark.timeout(900)
@pytest.mark.parametrize("n_states,S", [(128, 128), (170, 96)])
def test_qkv_product_writing_attention_operands_matches_two_step_path(n_states, S):
    """Uniform batches at head_dim 128 with enough rows for the 128 x 256 tile: the q | k | v product writes the
    attention kernel's operands itself (rotated q and k fragments, transposed v) instead of fp32 rows.  The same
    states through calls too small for that path (one state per call), and through the back-to-back layout,
    take the two-step path (fp32 rows, pack kernel): every bit of the pooled output must agree.  170 states of
    96 tokens end in a tile with two of its four 32-row blocks and put state boundaries inside tiles."""
    from paper_2604_24273_amd import runtime as R
    shape = synth.tiny_shape(n_layers=2, d=256, n_heads=4, n_kv_heads=2, head_dim=128, f=512, vocab=300,
                             rope_theta=500000.0)
    host = []
    enc = R.EncoderHandle(shape, seed=5, layer_sink=lambda l, w: host.append(w))
    ids = synth.token_ids(5, 500, (n_states, S), shape.vocab)
    print("fused q|k|v epilogue: %d states x %d tokens" % (n_states, S), flush=True)
    h = enc.forward(R.dev(ids))
    assert torch.equal(h, enc.forward(R.dev(ids)))
    for b in (0, 1, n_states // 2, n_states - 1):
        one = enc.forward(R.dev(ids[b:b + 1]))
        assert torch.equal(h[b:b + 1], one), b
    cu = (np.arange(n_states + 1) * S).astype(np.int32)
    hp = enc.forward_packed(R.dev(ids.reshape(-1).astype(np.int32)), cu, max_len=S)
    assert torch.equal(h, hp)
    cfg = O.EncoderConfig(shape.n_layers, shape.d, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.f,
                          shape.vocab, shape.rope_theta)
    sample = [0, n_states - 1]
    h_ref = O.encoder_forward(ids[sample], synth.embedding_bf16(5, shape), _oracle_layers(host),
                              synth.final_norm_gain(5, shape), cfg)
    for j, b in enumerate(sample):
        c = _cos(h.cpu().numpy()[b], h_ref[j])
        print("state %d: cosine %.7f" % (b, c), flush=True)
        assert c >= 0.999


@pytest.mark.timeout(600)
def test_fused_qkv_path_replays_from_a_hip_graph():
    """The path above captured into a HIP graph (after one ordinary call of the same shapes): every replay, with
    other eager work and synchronisations between the replays, reproduces the eager result bit for bit."""
    from paper_2604_24273_amd import binding as B
    from paper_2604_24273_amd import runtime as R
    shape = synth.tiny_shape(n_layers=2, d=256, n_heads=4, n_kv_heads=2, head_dim=128, f=512, vocab=300,
                             rope_theta=500000.0)
    enc = R.EncoderHandle(shape, seed=6)
    ids = R.dev(synth.token_ids(6, 500, (128, 128), shape.vocab))
    other = R.dev(synth.token_ids(6, 501, (128, 128), shape.vocab))
    ws = R.Workspace(B.brl_encoder_workspace_bytes(enc.struct, 128, 128))
    h = torch.empty((128, shape.d), dtype=torch.float32, device="cuda")

    def call(x):
        B.encoder_forward(enc.struct, x, 128, 128, None, h, ws.buf)

    call(ids)
    torch.cuda.synchronize()
    want = h.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call(ids)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(ids)
    for k in range(4):
        call(other)                      # eager work on the same workspace and output in between
        torch.cuda.synchronize()
        assert not torch.equal(h, want)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(h, want), "replay %d differs from the eager result" % k
