"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle.

Integer stages (ternary codes, int8 activations, int32 accumulators) must be
bit-exact.  fp32 outputs of one BitLinear / RMSNorm / FFN stage must agree to
max relative error 1e-5; encoder outputs to cosine >= 0.999 per state.
Inputs are the seeded synthetic tensors of paper_2604_24273_amd.synth.
"""
import numpy as np
import pytest

from oracle import bitrl_oracle as O
from paper_2604_24273_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

REL = 1e-5


def _mods():
    from paper_2604_24273_amd import binding as B
    from paper_2604_24273_amd import runtime as R
    B.lib()       # fails loudly if the library has not been built
    return B, R


def assert_fp_close(got: np.ndarray, ref: np.ndarray, rel: float = REL):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape
    scale = np.abs(ref).max()
    if scale == 0:
        assert np.all(got == 0)
        return
    d = np.abs(got - ref)
    assert d.max() / scale <= rel, "max rel err %.3e" % (d.max() / scale)
    assert np.all(d <= rel * np.abs(ref) + 0.1 * rel * scale)


def cosine(a, b):
    a = np.asarray(a, np.float64).ravel(); b = np.asarray(b, np.float64).ravel()
    return float(a @ b / (np.linalg.norm(a) * np.linalg.norm(b)))


# ------------------------------------------------------------------ weights

@pytest.mark.parametrize("n,k", [(2048, 2048), (6912, 2560), (2560, 6912), (70, 200), (33, 8), (1, 128), (640, 2560)])
def test_quantize_weights_bit_exact(n, k):
    B, R = _mods()
    print("quantize_weights", n, k, flush=True)
    W = synth.normal(0, 1, (n, k), 0.02)
    codes_ref, beta_ref = O.ternary_quantize(W)
    pl = R.quantize_linear(W, want_codes=True)
    assert pl.packed.numel() == B.brl_packed_bytes(n, k)
    beta = pl.beta.cpu().numpy()[0]
    assert beta.view(np.uint32) == np.float32(beta_ref).view(np.uint32), (beta, beta_ref)
    assert np.array_equal(pl.codes.cpu().numpy(), codes_ref)
    out = torch.empty((n, k), dtype=torch.int8, device="cuda")
    B.brl_unpack_codes(pl.packed, n, k, out)
    assert np.array_equal(out.cpu().numpy(), codes_ref)
    # deterministic: a second run gives the same blob
    pl2 = R.quantize_linear(W)
    assert torch.equal(pl.packed, pl2.packed) and torch.equal(pl.beta, pl2.beta)


def test_quantize_weights_special_matrices():
    B, R = _mods()
    for W in (np.zeros((40, 136), np.float32),                       # all zero: beta = eps, codes 0
              np.array([[3, -3, 1, -1, 3, -3, 1, -1]] * 2, np.float32),   # |w| == tau ties when eps = 0
              synth.normal(9, 1, (64, 256), 0.02) * np.float32(1e-4)):  # tiny scale: eps matters
        for eps in (1e-5, 0.0):
            c_ref, b_ref = O.ternary_quantize(W, eps)
            pl = R.quantize_linear(W, eps=eps, want_codes=True)
            assert np.float32(pl.beta.cpu().numpy()[0]).view(np.uint32) == np.float32(b_ref).view(np.uint32)
            assert np.array_equal(pl.codes.cpu().numpy(), c_ref)
    bad = np.ones((8, 16), np.float32); bad[1, 2] = np.inf
    with pytest.raises(B.BitrlError) as ei:
        R.quantize_linear(bad)
    assert ei.value.status == B.BRL_EINVAL


# ---------------------------------------------------------------- BitLinear

def _run_bitlinear(B, R, pl, X, residual=None, taps=True):
    m, k = X.shape
    n = pl.n_out
    y = torch.empty((m, n), dtype=torch.float32, device="cuda")
    xq = torch.zeros((m, k), dtype=torch.int8, device="cuda") if taps else None
    am = torch.zeros((m,), dtype=torch.float32, device="cuda") if taps else None
    acc = torch.zeros((m, n), dtype=torch.int32, device="cuda") if taps else None
    ws = R.Workspace(B.brl_bitlinear_workspace_bytes(m, n, k))
    B.bitlinear_forward(pl.packed, pl.beta, n, k, X, m, 1e-5, y, residual, xq, am, acc, ws.buf)
    torch.cuda.synchronize()
    return y, xq, am, acc, ws


@pytest.mark.parametrize("m,n,k", [
    (16, 2048, 2048),     # single-layer config
    (1, 6912, 2560), (1, 2560, 6912), (2, 2560, 6912), (3, 200, 264), (4, 6912, 2560),   # GEMV path
    (5, 96, 128), (33, 200, 264), (64, 2560, 2560), (100, 640, 2560), (300, 1000, 520),
    (256, 6912, 2560), (257, 2560, 6912), (1100, 3200, 3200),
    (600, 2560, 6912), (1300, 1000, 4608),                       # few 128 x 128 tiles, long k: k-split launches (ragged N in the second)
    (200, 1000, 4608), (700, 264, 6912),                         # 64 x 32 tiles, k split inside the workgroup
    (2050, 8192, 264), (2048, 8200, 128),      # enough tiles for the 8-wavefront kernel, ragged edges
    (1024, 640, 2560), (1025, 640, 2560),      # last size of the one-workgroup-per-token quantiser, first of the one-wavefront-per-token one
    (1100, 64, 8640), (1030, 40, 8200),        # widest rows of the one-wavefront-per-token quantiser (34 chunks), ragged k
    (2100, 64, 6912), (6200, 32, 2560),        # 16-token groups (past 2048 tokens at 6912 wide, past 6144 at 2560 wide)
    (1100, 40, 9216),                          # the widest rows supported: four wavefronts per token
])
def test_bitlinear_forward_parity(m, n, k):
    B, R = _mods()
    print("bitlinear_forward", m, n, k, flush=True)
    case = synth.bitlinear_case(0, n, k, m)
    if m >= 3:
        case["X"][1] = 0.0                      # an all-zero token must give an all-zero row
        case["X"][2] *= np.float32(1e-7)        # a tiny token exercises the absmax floor
    codes, beta = O.ternary_quantize(case["W"])
    taps = {}
    y_ref = O.bitlinear_forward(case["X"], codes, beta, taps=taps)
    pl = R.quantize_linear(case["W"])
    y, xq, am, acc, _ = _run_bitlinear(B, R, pl, R.dev(case["X"]))
    assert np.array_equal(xq.cpu().numpy(), taps["xq"])
    assert np.array_equal(am.cpu().numpy().view(np.uint32), taps["absmax"].view(np.uint32))
    assert np.array_equal(acc.cpu().numpy(), taps["acc"])
    assert_fp_close(y.cpu().numpy(), y_ref)
    assert np.array_equal(y.cpu().numpy(), y_ref)          # same fp32 op order: identical in practice
    if m >= 3:
        assert np.all(y.cpu().numpy()[1] == 0)


def test_bitlinear_forward_shape_sweep():
    """Seeded random shapes across the dispatch boundaries (1-4 token path, 16- and 8-wavefront k-split tiles,
    k-split tile launches, narrow and wide LDS tiles): integer stages exact, outputs identical, with and
    without the taps (the two epilogue families) and with a residual."""
    B, R = _mods()
    rng = np.random.default_rng(20241)
    shapes = []
    for _ in range(28):
        m = int(rng.choice([rng.integers(1, 9), rng.integers(9, 200), rng.integers(200, 1400)]))
        n = int(rng.choice([rng.integers(1, 97), 32 * rng.integers(1, 130), rng.integers(97, 3000)]))
        k = 8 * int(rng.choice([rng.integers(1, 48), rng.integers(48, 400), rng.integers(400, 1153)]))
        shapes.append((m, n, k))
    for idx, (m, n, k) in enumerate(shapes):
        print("bitlinear_forward sweep", m, n, k, flush=True)
        case = synth.bitlinear_case(1000 + idx, n, k, m)
        codes, beta = O.ternary_quantize(case["W"])
        taps = {}
        y_ref = O.bitlinear_forward(case["X"], codes, beta, taps=taps)
        pl = R.quantize_linear(case["W"])
        x = R.dev(case["X"])
        y, xq, am, acc, ws = _run_bitlinear(B, R, pl, x)
        assert np.array_equal(xq.cpu().numpy(), taps["xq"]), (m, n, k)
        assert np.array_equal(acc.cpu().numpy(), taps["acc"]), (m, n, k)
        assert np.array_equal(y.cpu().numpy(), y_ref), (m, n, k)
        res = synth.normal(1000 + idx, 7, (m, n))
        y2 = R.dev(res)
        B.bitlinear_forward(pl.packed, pl.beta, n, k, x, m, 1e-5, y2, y2, None, None, None, ws.buf)
        assert np.array_equal(y2.cpu().numpy(), O.bitlinear_forward(case["X"], codes, beta, residual=res)), (m, n, k)


@pytest.mark.parametrize("m", [1, 4, 48])
def test_bitlinear_residual_bf16_and_no_taps(m):
    B, R = _mods()
    n, k = 320, 384
    case = synth.bitlinear_case(3, n, k, m)
    xb = synth.to_bf16_bits(case["X"])
    x32 = synth.bf16_bits_to_f32(xb)
    res = synth.normal(3, 7, (m, n))
    codes, beta = O.ternary_quantize(case["W"])
    y_ref = O.bitlinear_forward(x32, codes, beta, residual=res)
    pl = R.quantize_linear(case["W"])
    y, *_ = _run_bitlinear(B, R, pl, R.bf16_from_bits(xb), residual=R.dev(res), taps=False)
    assert np.array_equal(y.cpu().numpy(), y_ref)


def test_gemv_pair_decode_shape_repeated():
    """x[1, d] -> up -> (re-quantised) -> down, many calls on one workspace: identical every time."""
    B, R = _mods()
    c = synth.gemv_pair_case(0)
    up_c, up_b = O.ternary_quantize(c["W_up"]); dn_c, dn_b = O.ternary_quantize(c["W_down"])
    h_ref = O.bitlinear_forward(c["x"], up_c, up_b)
    y_ref = O.bitlinear_forward(h_ref, dn_c, dn_b)
    up, dn = R.quantize_linear(c["W_up"]), R.quantize_linear(c["W_down"])
    x = R.dev(c["x"])
    d, f = 2560, 6912
    h = torch.empty((1, f), dtype=torch.float32, device="cuda")
    y = torch.empty((1, d), dtype=torch.float32, device="cuda")
    ws = R.Workspace(max(B.brl_bitlinear_workspace_bytes(1, f, d), B.brl_bitlinear_workspace_bytes(1, d, f)))
    outs = []
    for it in range(50):
        B.bitlinear_forward(up.packed, up.beta, f, d, x, 1, 1e-5, h, None, None, None, None, ws.buf)
        B.bitlinear_forward(dn.packed, dn.beta, d, f, h, 1, 1e-5, y, None, None, None, None, ws.buf)
        if it in (0, 1, 49):
            outs.append((h.cpu().numpy().copy(), y.cpu().numpy().copy()))
    for hh, yy in outs:
        assert np.array_equal(hh, h_ref)
        assert np.array_equal(yy, y_ref)


@pytest.mark.parametrize("m,n,k,count,bf16", [(1, 6912, 2560, 9, False), (1, 2560, 6912, 7, False), (3, 100, 200, 5, True),
                                              (2, 264, 8200, 3, False), (4, 96, 128, 700, False),
                                              # so many row blocks per workgroup that a wavefront stores its parked
                                              # results more than once per problem
                                              (4, 400000, 128, 1, False), (2, 300100, 256, 2, True)])
def test_bitlinear_forward_batch(m, n, k, count, bf16):
    """Many independent few-token problems in one launch: each equals the oracle and the one-problem entry point."""
    B, R = _mods()
    n_w = min(count, 4)                       # weights and inputs repeat across the batch, outputs do not
    cases = [synth.bitlinear_case(100 + i, n, k, m) for i in range(n_w)]
    pls = [R.quantize_linear(c["W"]) for c in cases]
    xs_host = [synth.bf16_bits_to_f32(synth.to_bf16_bits(c["X"])) if bf16 else c["X"] for c in cases]
    xs = [R.bf16_from_bits(synth.to_bf16_bits(c["X"])) if bf16 else R.dev(c["X"]) for c in cases]
    ys = [torch.full((m, n), float("nan"), dtype=torch.float32, device="cuda") for _ in range(count)]
    order = [(3 * i + 1) % n_w for i in range(count)]

    def ptrs(ts):
        return torch.tensor([t.data_ptr() for t in ts], dtype=torch.int64, device="cuda")

    B.bitlinear_forward_batch(ptrs([pls[j].packed for j in order]), ptrs([pls[j].beta for j in order]), n, k,
                              ptrs([xs[j] for j in order]), B.BRL_BF16 if bf16 else B.BRL_F32, m, 1e-5, ptrs(ys), count)
    torch.cuda.synchronize()
    refs = []
    for j in range(n_w):
        codes, beta = O.ternary_quantize(cases[j]["W"])
        refs.append(O.bitlinear_forward(xs_host[j], codes, beta))
    ws = R.Workspace(B.brl_bitlinear_workspace_bytes(m, n, k))
    single = []
    for j in range(n_w):
        y1 = torch.empty((m, n), dtype=torch.float32, device="cuda")
        B.bitlinear_forward(pls[j].packed, pls[j].beta, n, k, xs[j], m, 1e-5, y1, None, None, None, None, ws.buf)
        single.append(y1.cpu().numpy())
    for i in range(count):
        got = ys[i].cpu().numpy()
        assert np.array_equal(got, single[order[i]]), i
        assert_fp_close(got, refs[order[i]])
    # an empty batch is a no-op
    B.bitlinear_forward_batch(ptrs(ys[:1]), ptrs(ys[:1]), n, k, ptrs(ys[:1]), B.BRL_F32, m, 1e-5, ptrs(ys[:1]), 0)


# ---------------------------------------------------------------------- FFN

@pytest.mark.parametrize("m,d,f,bf16", [(256, 2560, 6912, True), (37, 256, 392, False), (3, 128, 264, True), (130, 3200, 8640, False),
                                        (160, 256, 4224, False), (160, 4224, 512, False),    # k-split down / k-split gate|up (GLU)
                                        # norms inside the one-wavefront-per-token quantiser: 34, 27 and 10 chunks per row,
                                        # groups of 8 tokens and (2100 at 6912 wide, 6200 at 2560 wide) of 16
                                        (1100, 128, 8640, False), (1100, 96, 6912, False), (2100, 96, 6912, False),
                                        (1200, 2560, 640, True), (6200, 2560, 64, False),
                                        (1100, 64, 9000, False)])      # four wavefronts per token, ragged k
def test_ffn_block_parity(m, d, f, bf16):
    B, R = _mods()
    print("ffn_block_forward", m, d, f, flush=True)
    c = synth.ffn_case(0, m, d, f)
    x32 = synth.bf16_bits_to_f32(c["x_bf16"]) if bf16 else synth.normal(0, 26, (m, d))
    w = O.FFNWeights(c["norm_g"], O.TernaryLinear.from_fp32(c["W_gate"]), O.TernaryLinear.from_fp32(c["W_up"]),
                     c["subln_g"], O.TernaryLinear.from_fp32(c["W_down"]))
    y_ref = O.ffn_block_forward(x32, w)
    hnd = R.FFNHandle(c["norm_g"], c["W_gate"], c["W_up"], c["subln_g"], c["W_down"])
    x = R.bf16_from_bits(c["x_bf16"]) if bf16 else R.dev(x32)
    y = torch.empty((m, d), dtype=torch.float32, device="cuda")
    ws = R.Workspace(B.brl_ffn_workspace_bytes(m, d, f))
    B.ffn_block_forward(hnd.struct, x, m, d, f, 1e-5, 1e-5, y, ws.buf)
    got = y.cpu().numpy()
    assert_fp_close(got, y_ref)
    # run again on the same workspace: bit-identical
    y2 = torch.empty_like(y)
    B.ffn_block_forward(hnd.struct, x, m, d, f, 1e-5, 1e-5, y2, ws.buf)
    assert torch.equal(y, y2)


# ------------------------------------------------------------------ encoder

def _oracle_encoder(shape, seed, layers_host):
    cfg = O.EncoderConfig(shape.n_layers, shape.d, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.f,
                          shape.vocab, shape.rope_theta)
    T = O.TernaryLinear.from_fp32
    layers = []
    for w in layers_host:
        layers.append(O.LayerWeights(w["attn_norm_g"], T(w["Wq"]), T(w["Wk"]), T(w["Wv"]), w["attn_subln_g"], T(w["Wo"]),
                                     O.FFNWeights(w["ffn_norm_g"], T(w["W_gate"]), T(w["W_up"]), w["ffn_subln_g"], T(w["W_down"]))))
    return cfg, layers


@pytest.mark.parametrize("kw,b,s", [
    (dict(n_layers=2, d=256, n_heads=4, n_kv_heads=2, head_dim=64, f=384, vocab=512), 5, 40),
    (dict(n_layers=3, d=128, n_heads=8, n_kv_heads=2, head_dim=16, f=264, vocab=300), 3, 70),
    (dict(n_layers=2, d=200, n_heads=2, n_kv_heads=2, head_dim=100, f=392, vocab=64), 2, 33),
    (dict(n_layers=1, d=256, n_heads=2, n_kv_heads=1, head_dim=128, f=512, vocab=1000), 4, 130),
    (dict(n_layers=2, d=64, n_heads=2, n_kv_heads=1, head_dim=32, f=128, vocab=50), 1, 1),
    (dict(n_layers=1, d=128, n_heads=4, n_kv_heads=4, head_dim=32, f=264, vocab=300), 2, 300),   # long multi-head states
    # states of at most 32 tokens: the one-kernel attention path
    (dict(n_layers=2, d=256, n_heads=4, n_kv_heads=2, head_dim=64, f=384, vocab=512), 5, 27),
    (dict(n_layers=2, d=200, n_heads=2, n_kv_heads=2, head_dim=100, f=392, vocab=64), 3, 32),
    (dict(n_layers=1, d=256, n_heads=2, n_kv_heads=1, head_dim=128, f=512, vocab=1000), 4, 19),
    (dict(n_layers=2, d=128, n_heads=8, n_kv_heads=1, head_dim=16, f=264, vocab=300), 2, 9),     # eight heads per k/v head
    (dict(n_layers=1, d=256, n_heads=8, n_kv_heads=8, head_dim=32, f=264, vocab=300), 3, 31),
])
@pytest.mark.parametrize("attn", ["mfma", "f32"])
def test_encoder_small_shapes(kw, b, s, attn):
    B, R = _mods()
    print("encoder_forward", kw, b, s, attn, flush=True)
    shape = synth.tiny_shape(**kw)
    host = []
    enc = R.EncoderHandle(shape, seed=1, layer_sink=lambda l, w: host.append(w),
                          attn_precision=B.BRL_ATTN_MFMA if attn == "mfma" else B.BRL_ATTN_F32)
    cfg, layers = _oracle_encoder(shape, 1, host)
    ids = synth.token_ids(1, 500, (b, s), shape.vocab)
    lengths = synth.state_lengths(1, 501, b, 1, s)
    emb = synth.embedding_bf16(1, shape)
    gfin = synth.final_norm_gain(1, shape)
    for ln in (None, lengths):
        h_ref = O.encoder_forward(ids, emb, layers, gfin, cfg, lengths=ln)
        h = enc.forward(R.dev(ids), None if ln is None else R.dev(ln)).cpu().numpy()
        for i in range(b):
            assert cosine(h[i], h_ref[i]) >= 0.999, (i, cosine(h[i], h_ref[i]))
        # An extra guard, not the bar: fp32-grade attention against fp64 attention differs in the last bits,
        # and where that flips one int8 rounding decision downstream the element moves by about 1/127 of its
        # token's absmax share, so no element-wise bound follows from the arithmetic; 5e-3 of the largest
        # output holds with a margin of two on every seeded case here.
        print("   guard ratio %.3e" % (np.abs(h - h_ref).max() / np.abs(h_ref).max()), flush=True)
        assert np.abs(h - h_ref).max() / np.abs(h_ref).max() < 5e-3
    # batch invariance and determinism, bit for bit
    h_all = enc.forward(R.dev(ids))
    assert torch.equal(h_all, enc.forward(R.dev(ids)))
    if b > 1:
        h_one = enc.forward(R.dev(ids[1:2]))
        assert torch.equal(h_all[1:2], h_one)


@pytest.mark.parametrize("kw,lens", [
    (dict(n_layers=2, d=256, n_heads=4, n_kv_heads=2, head_dim=64, f=384, vocab=512), [15, 40, 1, 32, 33, 27, 64, 31]),
    (dict(n_layers=2, d=200, n_heads=2, n_kv_heads=2, head_dim=100, f=392, vocab=64), [7, 70, 36]),
    (dict(n_layers=1, d=256, n_heads=8, n_kv_heads=2, head_dim=32, f=512, vocab=1000), [5]),
    (dict(n_layers=1, d=128, n_heads=2, n_kv_heads=1, head_dim=128, f=264, vocab=300), [129, 2, 96, 18, 40]),
    (dict(n_layers=2, d=256, n_heads=4, n_kv_heads=1, head_dim=64, f=384, vocab=512), [15, 27, 1, 32, 8]),   # all short
    (dict(n_layers=1, d=256, n_heads=2, n_kv_heads=2, head_dim=128, f=264, vocab=300), [27]),
])
@pytest.mark.parametrize("attn", ["mfma", "f32"])
def test_encoder_packed_variable_length(kw, lens, attn):
    """States of different lengths stored back to back: every state equals the oracle run on that state
    alone, and (bit for bit) the padded entry point with `lengths`."""
    B, R = _mods()
    print("encoder_forward_packed", kw, lens, attn, flush=True)
    shape = synth.tiny_shape(**kw)
    host = []
    enc = R.EncoderHandle(shape, seed=2, layer_sink=lambda l, w: host.append(w),
                          attn_precision=B.BRL_ATTN_MFMA if attn == "mfma" else B.BRL_ATTN_F32)
    cfg, layers = _oracle_encoder(shape, 2, host)
    emb = synth.embedding_bf16(2, shape)
    gfin = synth.final_norm_gain(2, shape)
    nb, smax = len(lens), max(lens)
    padded = synth.token_ids(2, 500, (nb, smax), shape.vocab)
    flat = np.concatenate([padded[i, :n] for i, n in enumerate(lens)]).astype(np.int32)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    h = enc.forward_packed(R.dev(flat), cu)
    # a larger bound on the lengths changes nothing
    assert torch.equal(h, enc.forward_packed(R.dev(flat), cu, max_len=smax + 29))
    h_pad = enc.forward(R.dev(padded), R.dev(np.asarray(lens, dtype=np.int32)))
    assert torch.equal(h, h_pad)
    hn = h.cpu().numpy()
    for i, n in enumerate(lens):
        h_ref = O.encoder_forward(padded[i:i + 1, :n], emb, layers, gfin, cfg)[0]
        assert cosine(hn[i], h_ref) >= 0.999, (i, n, cosine(hn[i], h_ref))
        print("   guard ratio %.3e" % (np.abs(hn[i] - h_ref).max() / np.abs(h_ref).max()), flush=True)
        assert np.abs(hn[i] - h_ref).max() / np.abs(h_ref).max() < 5e-3


def test_head_parity_and_variants():
    B, R = _mods()
    for hidden, act in (((256,), B.BRL_ACT_TANH), ((256, 128), B.BRL_ACT_TANH), ((64,), B.BRL_ACT_RELU), ((), B.BRL_ACT_TANH)):
        shape = synth.tiny_shape(d=2560, head_hidden=hidden, n_actions=18)
        hh = R.HeadHandle(shape, seed=0, act=act)
        h = synth.normal(0, 400, (64, 2560))
        logits, value = hh.forward(R.dev(h))
        name = "tanh" if act == B.BRL_ACT_TANH else "relu"
        lr, vr = O.policy_value_head(h, O.MLP(*hh.host["policy"], name), O.MLP(*hh.host["value"], name))
        assert_fp_close(logits.cpu().numpy(), lr)
        assert_fp_close(value.cpu().numpy(), vr)
        p = O.softmax(logits.cpu().numpy())
        assert np.allclose(p.sum(axis=1), 1.0)


def test_entry_points_replay_from_a_hip_graph():
    """encoder_forward_packed + policy_value_head enqueue kernels only: captured once (after one ordinary call),
    every replay - with eager calls and synchronisations in between - reproduces the eager result bit for bit."""
    B, R = _mods()
    shape = synth.tiny_shape(n_layers=2, d=128, n_heads=4, n_kv_heads=2, head_dim=32, f=264, vocab=300,
                             n_actions=6, head_hidden=(32,))
    enc = R.EncoderHandle(shape, seed=3)
    head = R.HeadHandle(shape, seed=3)
    lens = [17, 40, 5]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    ids = R.dev(synth.token_ids(3, 500, (int(cu[-1]),), shape.vocab))
    cu_dev = R.dev(cu)
    ws = R.Workspace(B.brl_encoder_packed_workspace_bytes(enc.struct, 3, int(cu[-1]), 40))
    hws = R.Workspace(B.brl_head_workspace_bytes(head.struct, 3))
    h = torch.empty((3, shape.d), dtype=torch.float32, device="cuda")
    logits = torch.empty((3, 6), dtype=torch.float32, device="cuda")
    value = torch.empty((3,), dtype=torch.float32, device="cuda")

    def call():
        B.encoder_forward_packed(enc.struct, ids, cu_dev, cu, 3, 40, h, ws.buf)
        B.policy_value_head(head.struct, h, 3, logits, value, hws.buf)

    call()
    torch.cuda.synchronize()
    ref = (h.clone(), logits.clone(), value.clone())
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call()
    for _ in range(4):
        h.zero_(); logits.zero_(); value.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(h, ref[0]) and torch.equal(logits, ref[1]) and torch.equal(value, ref[2])
        call()                               # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(h, ref[0])
