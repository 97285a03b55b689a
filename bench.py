#!/usr/bin/env python3
"""Benchmark of the frozen ternary-encoder hot path on one MI355X.

One step = one pass of the whole hot path over one batch of seeded synthetic
states: token ids -> embedding -> 30 x (RMSNorm, int8 quant, q|k|v BitLinear,
rotary causal GQA attention, subLN, o BitLinear, RMSNorm, gate|up BitLinear,
squared-ReLU GLU, subLN, down BitLinear) -> final norm -> mean-pool -> fp32
policy / value heads, at the 2B BitNet shape with 64 states x 128 tokens.
Weights, embedding and ids are resident in HBM before the timed region.

Prints ONE JSON line.  Besides the headline states/s it carries the roofline
of the dominant kernel (the int8 MFMA GEMM, durations from HIP events recorded
by the library around every launch in a second, identically sized region), the
1-token GEMV pair figures (one launch per product, and the whole walk as two
batched launches), the latency of one short state per call, one PPO update of
the heads, and the CPU oracle timed on a bounded sample as context.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0      # MI355X dense int8, TOP/s
HBM_PEAK_GBS = 8000.0             # MI355X HBM3E, GB/s
# timing classes of the library that are BitLinear matrix products (the last: the wide tile on the q | k | v product,
# with the epilogue that writes the attention kernel's operands)
GEMM_CLASSES = ("gemm", "gemm_narrow", "gemm_qkv_attn")


# HBM bytes per launch from rocprofv3 counters (FETCH_SIZE + WRITE_SIZE, each scaled by what the same counter
# reads for a copy kernel of known size).  These are NOT measured by a bench run: each entry names the profile
# summary it was copied from and the kernel it refers to, and is reset to None whenever that kernel changes
# until the counters have been taken again.
ROOFLINE_TRAFFIC = {
    # FETCH_SIZE 114 010 KiB x 2.0 + WRITE_SIZE 221 184 KiB x 1.0 per gate|up launch (the only product of the 2B
    # step that runs this kernel since the q | k | v product has its own); algorithmic: 21 + 8.8 MB in, 226.5 MB out
    "encoder-2b": {"bytes": 460.0e6, "kernel": "gemm_lds_kernel<2,2,2,4>",
                   "source": "profiles/bench_encoder_2b_hbm_traffic_counters.txt"},
    "prefill-3b": {"bytes": None, "kernel": "gemm_lds_kernel<2,2,2,4>", "source": None},
    "rl-states-2b": {"bytes": None, "kernel": "gemm_lds_kernel<2,2,2,4>", "source": None},
}
# batched GEMV: fetched bytes (FETCH_SIZE x 2.0; the outputs, 0.4 % of the bytes, are not in it) / algorithmic bytes
# per launch, from the same kind of counter run with one pair of weight buffers per product, as in the timed leg
# (256 products per launch: 1132.8 MB and 1139.9 MB fetched by the two kinds of launch against 2 x 1138.5 MB)
GEMV_BATCH_FETCH = {"ratio": 0.998, "source": "profiles/bench_encoder_2b_hbm_traffic_counters.txt"}


def linear_macs_per_token(shape) -> int:
    dq = shape.n_heads * shape.head_dim
    dkv = shape.n_kv_heads * shape.head_dim
    per_layer = shape.d * (dq + 2 * dkv) + dq * shape.d + 2 * shape.f * shape.d + shape.d * shape.f
    return per_layer * shape.n_layers


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", choices=["encoder-2b", "prefill-3b", "rl-states-2b"], default="encoder-2b",
                    help="encoder-2b: 64 states x 128 tokens at the 2B shape (the headline); "
                         "prefill-3b: 1024 states x 512 tokens at the 3B shape (large-batch regime); "
                         "rl-states-2b: 1024 states of 15-40 tokens each at the 2B shape, stored back to back")
    ap.add_argument("--states", type=int, default=None)
    ap.add_argument("--tokens", type=int, default=None)
    ap.add_argument("--layers", type=int, default=None, help="debug only: fewer layers (invalidates the metric)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-gemv", action="store_true")
    ap.add_argument("--no-ppo", action="store_true")
    ap.add_argument("--no-single-state", action="store_true")
    ap.add_argument("--no-critics", action="store_true", help="skip the int8-weight critic encoder and ensemble legs")
    ap.add_argument("--no-layer", action="store_true", help="skip the single 16 x 2048 x 2048 BitLinear layer leg")
    ap.add_argument("--no-ffn", action="store_true", help="skip the 256-token FFN block leg")
    ap.add_argument("--no-prefill-3b", action="store_true", help="skip the 3B-shape 64 x 512 micro-batch leg")
    ap.add_argument("--no-vendor-gemm", action="store_true",
                    help="skip the context leg that times the vendor int8 GEMM (torch._int_mm) on the same layer shapes")
    ap.add_argument("--gemv-pool", type=int, default=None,
                    help="distinct weight-pair buffers the GEMV legs walk (default: one per call, so that a batched "
                         "launch reads every weight byte exactly once and nothing can come out of a cache)")
    ap.add_argument("--cpu-sample-states", type=int, default=6,
                    help="states of the batch the CPU oracle is timed on (about 2 s each on 16 cores)")
    ap.add_argument("--gemv-calls", type=int, default=1000)
    ap.add_argument("--streams", type=int, default=1,
                    help="extra leg: also time the batch as this many concurrent micro-batches on separate HIP streams")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on ONE GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2604_24273_amd import binding as B
    from paper_2604_24273_amd import build as BUILD
    from paper_2604_24273_amd import runtime as R
    from paper_2604_24273_amd import synth

    if not os.path.exists(B.LIB_PATH):
        BUILD.build()
    B.lib()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)

    packed = args.workload == "rl-states-2b"
    shape = synth.SHAPE_3B if args.workload == "prefill-3b" else synth.SHAPE_2B
    n_layers = shape.n_layers if args.layers is None else args.layers
    Bn = args.states if args.states is not None else (64 if args.workload == "encoder-2b" else 1024)
    S = args.tokens if args.tokens is not None else {"encoder-2b": 128, "prefill-3b": 512, "rl-states-2b": 40}[args.workload]
    want_cpu = not args.no_cpu_baseline

    # ---- weights: seeded host draws -> packed on the GPU; the oracle's copy is quantised on the side
    oracle_jobs = []
    pool = ThreadPoolExecutor(max_workers=4) if want_cpu else None
    if want_cpu:
        from oracle import bitrl_oracle as O

        def _oracle_layer(w):
            T = O.TernaryLinear.from_fp32
            return O.LayerWeights(w["attn_norm_g"], T(w["Wq"]), T(w["Wk"]), T(w["Wv"]), w["attn_subln_g"], T(w["Wo"]),
                                  O.FFNWeights(w["ffn_norm_g"], T(w["W_gate"]), T(w["W_up"]), w["ffn_subln_g"],
                                               T(w["W_down"])))

    def sink(l, w):
        if want_cpu:
            oracle_jobs.append(pool.submit(_oracle_layer, w))

    t0 = time.time()
    want_critics = not args.no_critics and args.workload == "encoder-2b"
    enc = R.EncoderHandle(shape, seed=0, layer_sink=sink, n_layers=n_layers, int8_twin=want_critics)
    head = R.HeadHandle(shape, seed=0)
    ids_host = synth.token_ids(0, 500, (Bn, S), shape.vocab)
    if packed:
        # states of 15 .. S tokens (the paper's serialised states are 15-40 tokens), stored back to back
        lens = synth.state_lengths(0, 501, Bn, min(15, S), S)
        cu_host = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        ids = R.dev(np.concatenate([ids_host[i, :n] for i, n in enumerate(lens)]).astype(np.int32))
        cu_dev = R.dev(cu_host)
        tokens_step = int(cu_host[-1])
        enc.ws = R.Workspace(B.brl_encoder_packed_workspace_bytes(enc.struct, Bn, tokens_step, S))
        h_buf = torch.empty((Bn, shape.d), dtype=torch.float32, device="cuda")

        def encode():
            B.encoder_forward_packed(enc.struct, ids, cu_dev, cu_host, Bn, S, h_buf, enc.ws.buf)
            return h_buf
    else:
        lens = np.full((Bn,), S, dtype=np.int32)
        ids = R.dev(ids_host)
        tokens_step = Bn * S

        def encode():
            return enc.forward(ids)
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    def step():
        return head.forward(encode())

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3
    states_per_s = Bn / (ms_per_step / 1e3)

    # ---- per-kernel durations: same region again with the library's event timing on
    B.brl_timing_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    B.brl_timing_enable(False)
    classes = {}
    for kc, name in enumerate(B.KERNEL_CLASSES):
        n, ms, ops = B.brl_timing_read_ops(kc)
        classes[name] = {"launches_per_step": n / args.steps, "ms_per_step": ms / args.steps,
                         "int8_ops_per_step": ops / args.steps}
    macs_tok = linear_macs_per_token(shape) * n_layers // shape.n_layers
    ops_step = 2.0 * macs_tok * tokens_step
    # dominant kernel: the 128 x 256-tile int8 MFMA GEMM; its algorithmic ops per launch are the
    # 2 M N K of the products it ran (counted by the library per launch), over its own event time
    gemm = classes["gemm"]
    gemm_launches = max(gemm["launches_per_step"], 1)
    gemm_avg_ms = gemm["ms_per_step"] / gemm_launches
    ops_per_launch = gemm["int8_ops_per_step"] / gemm_launches
    achieved_tops = ops_per_launch / (gemm_avg_ms * 1e-3) / 1e12 if gemm_avg_ms > 0 else 0.0
    all_gemm_ms = sum(classes[c]["ms_per_step"] for c in GEMM_CLASSES)
    all_gemm_ops = sum(classes[c]["int8_ops_per_step"] for c in GEMM_CLASSES)
    roofline = {"bound": "mfma", "kernel": "gemm_lds_kernel<2,2,2,4> (int8 MFMA BitLinear, 128x256 tile)",
                "achieved": round(achieved_tops, 2), "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                "frac": round(achieved_tops / INT8_MFMA_PEAK_TOPS, 4), "traffic": ROOFLINE_TRAFFIC[args.workload]["bytes"],
                "traffic_source": ROOFLINE_TRAFFIC[args.workload]["source"],
                "avg_launch_ms": round(gemm_avg_ms, 5), "launches_per_step": gemm_launches,
                "ops_per_launch": ops_per_launch,
                "all_bitlinear_gemms": {"ms_per_step": round(all_gemm_ms, 4),
                                        "tops": round(all_gemm_ops / (all_gemm_ms * 1e-3) / 1e12, 2) if all_gemm_ms > 0 else 0.0,
                                        "ops_counted_vs_analytic": round(all_gemm_ops / ops_step, 6)}}

    # ---- optional extra leg: the same batch as concurrent micro-batches on separate streams
    concurrent = None
    if args.streams > 1 and not packed:
        parts = [p.contiguous() for p in torch.chunk(ids, args.streams, dim=0)]
        wss = [R.Workspace(B.brl_encoder_workspace_bytes(enc.struct, p.shape[0], S)) for p in parts]
        h_all = torch.empty((Bn, shape.d), dtype=torch.float32, device="cuda")
        hs = list(torch.split(h_all, [p.shape[0] for p in parts], dim=0))     # contiguous row slices
        sts = [torch.cuda.Stream() for _ in parts]

        def cstep():
            main = torch.cuda.current_stream()
            for p, w, hh, st in zip(parts, wss, hs, sts):
                st.wait_stream(main)
                with torch.cuda.stream(st):
                    B.encoder_forward(enc.struct, p, p.shape[0], S, None, hh, w.buf)
            for st in sts:
                main.wait_stream(st)
            return head.forward(h_all)

        for _ in range(args.warmup):
            cstep()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            cstep()
        torch.cuda.synchronize()
        cms = (time.perf_counter() - t0) / args.steps * 1e3
        same = bool(torch.equal(h_all, enc.forward(ids)))
        concurrent = {"streams": args.streams, "ms_per_step": round(cms, 4), "states_per_s": round(Bn / cms * 1e3, 1),
                      "bit_identical_to_single_call": same}

    # ---- 1-token GEMV pair (decode shape), 1000 calls
    gemv = None
    if not args.no_gemv:
        gemv = bench_gemv(torch, B, R, synth, args.gemv_calls, args.gemv_pool or args.gemv_calls)

    # ---- the single BitLinear layer (16 x 2048 x 2048) and the 256-token FFN block of the workload list
    layer = None
    if not args.no_layer and args.workload == "encoder-2b":
        layer = bench_layer(torch, B, R, synth)
    ffn = None
    if not args.no_ffn and args.workload == "encoder-2b":
        ffn = bench_ffn(torch, B, R, synth)

    vendor = None
    if not args.no_vendor_gemm and args.workload == "encoder-2b":
        vendor = bench_vendor_gemm(torch, Bn * S, shape)

    # ---- one short state per call (the paper's deployment shape: a 15-40 token state per environment step)
    single = None
    if not args.no_gemv and not args.no_single_state and shape is synth.SHAPE_2B:
        single = bench_single_state(torch, B, R, synth, np, enc, head, shape)

    # ---- PPO update of the heads on a cached rollout (the step after the path)
    ppo = None
    if not args.no_ppo and shape is synth.SHAPE_2B:
        ppo = bench_ppo(torch, B, R, synth, np, shape, want_cpu)

    # ---- critic variants of the ablation: int8-weight backbone on the same batch, ensembles of value heads
    critics = None
    if want_critics:
        critics = bench_critics(torch, B, R, synth, enc, ids, Bn, S, shape, args.steps, args.warmup)

    # ---- CPU oracle on a bounded sample of the same workload
    cpu = None
    if want_cpu:
        from oracle import bitrl_oracle as O
        layers = [j.result() for j in oracle_jobs]
        pool.shutdown()
        cfg = O.EncoderConfig(n_layers, shape.d, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.f,
                              shape.vocab, shape.rope_theta)
        emb = synth.embedding_bf16(0, shape)
        gfin = synth.final_norm_gain(0, shape)
        pol = O.MLP(*head.host["policy"], "tanh")
        val = O.MLP(*head.host["value"], "tanh")
        ns = max(1, min(args.cpu_sample_states, Bn))
        t0 = time.perf_counter()
        if packed:
            h_ref = np.concatenate([O.encoder_forward(ids_host[i:i + 1, :lens[i]], emb, layers, gfin, cfg) for i in range(ns)])
        else:
            h_ref = O.encoder_forward(ids_host[:ns], emb, layers, gfin, cfg)
        l_ref, v_ref = O.policy_value_head(h_ref, pol, val)
        cpu_s = time.perf_counter() - t0
        h_gpu = encode()[:ns].cpu().numpy().astype(np.float64)
        cosines = [float(h_gpu[i] @ h_ref[i] / np.linalg.norm(h_gpu[i]) / np.linalg.norm(h_ref[i])) for i in range(ns)]
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        cpu = {"value": round(ns / cpu_s, 4), "unit": "states/s", "cores": int(cores), "kind": "oracle",
               "sample": "%d of the %d states (%s tokens each, all %d layers + heads), NumPy oracle, fp64 BLAS integer matmul"
                         % (ns, Bn, "/".join(str(int(n)) for n in lens[:ns]) if packed else str(S), n_layers),
               "seconds": round(cpu_s, 2), "min_cosine_gpu_vs_oracle": round(min(cosines), 6)}

    # ---- one 64-state x 512-token micro-batch of the 3B-shape prefill (1 of the 16 the 1024-state workload makes)
    prefill = None
    if not args.no_prefill_3b and args.workload == "encoder-2b":
        del enc
        torch.cuda.empty_cache()
        prefill = bench_prefill_3b(torch, B, R, synth, np)

    out = {
        "metric": "encoded RL states/sec at %s shape (BitLinear int8 TOPS as %% of roofline alongside)"
                  % ("3B" if args.workload == "prefill-3b" else "2B"),
        "value": round(states_per_s, 2), "unit": "states/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8 (ternary x int8 -> int32, fp32 rescale)", "data": "synthetic",
        "config": {"workload": "frozen %s-shape ternary encoder + fp32 heads: %d layers, hidden %d, %d/%d heads, FFN %d, "
                               "vocab %d; batch %d states x %s tokens, seed 0"
                               % ("3B" if args.workload == "prefill-3b" else "2B", n_layers, shape.d, shape.n_heads,
                                  shape.n_kv_heads, shape.f, shape.vocab, Bn,
                                  ("15-%d (uniform, %d in all, no padding)" % (S, tokens_step)) if packed else str(S)),
                   "states": Bn, "tokens_per_state": (tokens_step / Bn) if packed else S, "int8_ops_per_step": ops_step},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernel_classes_ms_per_step": {k: round(v["ms_per_step"], 4) for k, v in classes.items()},
        "linear_tops_wall": round(ops_step / (ms_per_step * 1e-3) / 1e12, 2),
        "int8_ceiling_states_per_s": round(Bn / (ops_step / (INT8_MFMA_PEAK_TOPS * 1e12)), 1),
        "bitlinear_layer_16x2048x2048": layer,
        "ffn_block_256_tokens": ffn,
        "prefill_3b_microbatch": prefill,
        "vendor_int8_gemm_context": vendor,
        "gemv_pair": gemv,
        "single_state_latency": single,
        "ppo_head_update": ppo,
        "critic_variants": critics,
        "concurrent_microbatches": concurrent,
        "paper_context": {"hardware": "Raspberry Pi 4 (Cortex-A72 @ 1.5 GHz), bitnet.cpp", "steps_per_s": 40.3,
                          "median_latency_ms": 24.8, "note": "one 15-40 token state per step; context only"},
        "setup_seconds": round(setup_s, 1),
    }
    print(json.dumps(out))
    return 0


def _drain_timing(B):
    for k in range(len(B.KERNEL_CLASSES)):
        B.brl_timing_read(k)


def bench_layer(torch, B, R, synth, calls: int = 200):
    """One BitLinear layer, W 2048 x 2048 ~ N(0, 0.02) ternarised, X 16 x 2048 ~ N(0, 1) fp32 (seed 0): two launches
    (per-token quantisation, few-token MFMA kernel).  Far too small for either roofline (1 MB of weights, 0.13 GOP):
    a latency figure."""
    n = k = 2048
    m = 16
    c = synth.bitlinear_case(0, n, k, m)
    pl = R.quantize_linear(c["W"])
    x = R.dev(c["X"])
    y = torch.empty((m, n), dtype=torch.float32, device="cuda")
    ws = R.Workspace(B.brl_bitlinear_workspace_bytes(m, n, k))

    def call():
        B.bitlinear_forward(pl.packed, pl.beta, n, k, x, m, 1e-5, y, None, None, None, None, ws.buf)

    for _ in range(20):
        call()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(calls):
        call()
    torch.cuda.synchronize()
    wall_us = (time.perf_counter() - t0) / calls * 1e6
    _drain_timing(B)
    B.brl_timing_enable(True)
    for _ in range(calls):
        call()
    torch.cuda.synchronize()
    B.brl_timing_enable(False)
    nq, qms = B.brl_timing_read(B.BRL_KC_ACT_QUANT)
    ng, gms, ops = B.brl_timing_read_ops(B.BRL_KC_GEMM_NARROW)
    _drain_timing(B)
    gemm_us = gms / max(ng, 1) * 1e3
    return {"workload": "W 2048x2048 ternary, X 16x2048 fp32, seed 0", "calls": calls,
            "wall_us_per_call": round(wall_us, 3), "quant_kernel_us": round(qms / max(nq, 1) * 1e3, 3),
            "gemm_kernel_us": round(gemm_us, 3), "int8_ops": 2.0 * m * n * k,
            "gemm_tops": round(2.0 * m * n * k / (gemm_us * 1e-6) / 1e12, 3) if gemm_us > 0 else 0.0,
            "note": "latency bound: 1.05 MB of packed weights and 0.134 GOP are below 0.2 us at either roofline"}


def bench_ffn(torch, B, R, synth, calls: int = 200, m: int = 256, d: int = 2560, f: int = 6912):
    """One 2B-shape FFN block on 256 tokens: RMSNorm -> gate | up BitLinear -> squared-ReLU GLU -> sub-layer norm ->
    down BitLinear + residual, bf16-valued input (seed 0).  Whole-block time and the int8 rate over its GEMM
    launches (2 M (2 f d + d f) = 27.2 GOP)."""
    c = synth.ffn_case(0, m, d, f)
    h = R.FFNHandle(c["norm_g"], c["W_gate"], c["W_up"], c["subln_g"], c["W_down"])
    x = R.bf16_from_bits(c["x_bf16"])
    y = torch.empty((m, d), dtype=torch.float32, device="cuda")
    ws = R.Workspace(B.brl_ffn_workspace_bytes(m, d, f))

    def call():
        B.ffn_block_forward(h.struct, x, m, d, f, 1e-5, 1e-5, y, ws.buf)

    for _ in range(20):
        call()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(calls):
        call()
    torch.cuda.synchronize()
    wall_us = (time.perf_counter() - t0) / calls * 1e6
    _drain_timing(B)
    B.brl_timing_enable(True)
    for _ in range(calls):
        call()
    torch.cuda.synchronize()
    B.brl_timing_enable(False)
    per = {}
    gemm_ms, gemm_ops, gemm_n = 0.0, 0.0, 0
    for kc, name in enumerate(B.KERNEL_CLASSES):
        n, ms, ops = B.brl_timing_read_ops(kc)
        if n:
            per[name] = {"launches_per_call": n / calls, "us_per_call": round(ms / calls * 1e3, 3)}
        if name in GEMM_CLASSES:
            gemm_ms += ms
            gemm_ops += ops
            gemm_n += n
    gemm_us = gemm_ms / calls * 1e3
    tops = gemm_ops / calls / (gemm_us * 1e-6) / 1e12 if gemm_us > 0 else 0.0
    return {"workload": "RMSNorm(2560) -> gate|up 2560->6912 -> sq-ReLU GLU -> subLN(6912) -> down 6912->2560 + residual; "
                        "256 tokens, bf16-valued input, seed 0",
            "calls": calls, "wall_us_per_block": round(wall_us, 3), "kernel_classes": per,
            "gemm_us_per_block": round(gemm_us, 3), "gemm_launches_per_block": gemm_n / calls,
            "int8_ops_per_block": gemm_ops / calls,
            "roofline": {"bound": "mfma", "kernel": "the BitLinear GEMM launches of the block (gate|up with the GLU epilogue, down)",
                         "achieved": round(tops, 2), "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                         "frac": round(tops / INT8_MFMA_PEAK_TOPS, 4), "traffic": None}}


def bench_prefill_3b(torch, B, R, synth, np, states: int = 64, tokens: int = 512, steps: int = 5, warmup: int = 2):
    """The 3B-shape large-batch prefill, one micro-batch: 64 states x 512 tokens (32 768 token rows) is what one pass
    of encoder_forward works on at a time; the 1024-state workload is 16 of these back to back
    (`--workload prefill-3b` times all 16)."""
    shape = synth.SHAPE_3B
    t0 = time.time()
    enc = R.EncoderHandle(shape, seed=0)
    ids = R.dev(synth.token_ids(0, 500, (states, tokens), shape.vocab))
    torch.cuda.synchronize()
    setup_s = time.time() - t0
    for _ in range(warmup):
        enc.forward(ids)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        enc.forward(ids)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    _drain_timing(B)
    B.brl_timing_enable(True)
    for _ in range(steps):
        enc.forward(ids)
    torch.cuda.synchronize()
    B.brl_timing_enable(False)
    per = {}
    gemm_ms, gemm_ops = 0.0, 0.0
    for kc, name in enumerate(B.KERNEL_CLASSES):
        n, kms, ops = B.brl_timing_read_ops(kc)
        if n:
            per[name] = round(kms / steps, 3)
        if name in GEMM_CLASSES:
            gemm_ms += kms
            gemm_ops += ops
    ops_step = 2.0 * linear_macs_per_token(shape) * states * tokens
    tops = gemm_ops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    return {"workload": "3B shape: 26 layers, hidden 3200, 32 heads of 100, FFN 8640, vocab 32000; ONE micro-batch of "
                        "%d states x %d tokens (1 of the 16 micro-batches of the 1024-state prefill), seed 0" % (states, tokens),
            "steps": steps, "ms_per_microbatch": round(ms, 3), "states_per_s": round(states / ms * 1e3, 1),
            "int8_ops_per_microbatch": ops_step, "linear_tops_wall": round(ops_step / (ms * 1e-3) / 1e12, 2),
            "kernel_classes_ms": per,
            "roofline": {"bound": "mfma", "kernel": "all BitLinear GEMM launches of the micro-batch", "achieved": round(tops, 2),
                         "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s", "frac": round(tops / INT8_MFMA_PEAK_TOPS, 4),
                         "traffic": None},
            "setup_seconds": round(setup_s, 1)}


def bench_vendor_gemm(torch, M: int, shape):
    """Context only, not part of the library's path: the vendor's dense int8 GEMM (hipBLASLt behind torch._int_mm,
    int8 x int8 -> int32, no 2-bit decode, no rescale, no GLU) on the four BitLinear products of a 2B-shape layer,
    with operands distributed like the library's (int8 activations of sigma 36, ternary weights as int8)."""
    dq, dkv = shape.n_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    shapes = {"qkv": (dq + 2 * dkv, shape.d), "o": (shape.d, dq), "gate_up": (2 * shape.f, shape.d), "down": (shape.d, shape.f)}
    out = {}
    try:
        gen = torch.Generator(device="cuda")
        gen.manual_seed(0)
        for name, (N, K) in shapes.items():
            a = torch.clamp(torch.round(torch.randn((M, K), generator=gen, device="cuda") * 36.0), -127, 127).to(torch.int8)
            b = torch.randint(-1, 2, (K, N), generator=gen, device="cuda", dtype=torch.int8)
            for _ in range(3):
                torch._int_mm(a, b)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                torch._int_mm(a, b)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) / 10 * 1e3
            out[name] = {"M": M, "N": N, "K": K, "us": round(us, 1), "tops": round(2.0 * M * N * K / (us * 1e-6) / 1e12, 1)}
            del a, b
        tot_ops = sum(2.0 * v["M"] * v["N"] * v["K"] for v in out.values())
        tot_us = sum(v["us"] for v in out.values())
        out["all_four"] = {"us": round(tot_us, 1), "tops": round(tot_ops / (tot_us * 1e-6) / 1e12, 1)}
        out["note"] = "torch._int_mm (hipBLASLt), dense int8 weights; context for the library's BitLinear rate, not a target"
    except Exception as e:          # an unsupported build of torch must not fail the benchmark
        out = {"unavailable": str(e)[:160]}
    return out


def bench_single_state(torch, B, R, synth, np, enc, head, shape, n_tokens: int = 27, calls: int = 50):
    """encoder_forward_packed + heads on ONE state of n_tokens tokens per call: launch-per-kernel from the host,
    and the same call sequence captured once into a HIP graph and replayed (the entry points allocate nothing and
    never synchronise, so they can be captured as they are)."""
    ids = R.dev(synth.token_ids(0, 510, (n_tokens,), shape.vocab))
    cu_host = np.asarray([0, n_tokens], dtype=np.int32)
    cu_dev = R.dev(cu_host)
    ws = R.Workspace(B.brl_encoder_packed_workspace_bytes(enc.struct, 1, n_tokens, n_tokens))
    hws = R.Workspace(B.brl_head_workspace_bytes(head.struct, 1))
    h = torch.empty((1, shape.d), dtype=torch.float32, device="cuda")
    logits = torch.empty((1, head.n_actions), dtype=torch.float32, device="cuda")
    value = torch.empty((1,), dtype=torch.float32, device="cuda")

    def call():
        B.encoder_forward_packed(enc.struct, ids, cu_dev, cu_host, 1, n_tokens, h, ws.buf)
        B.policy_value_head(head.struct, h, 1, logits, value, hws.buf)

    for _ in range(5):
        call()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(calls):
        call()
    torch.cuda.synchronize()
    eager_ms = (time.perf_counter() - t0) / calls * 1e3
    ref = (h.clone(), logits.clone(), value.clone())

    graph_ms, same = None, None
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            call()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            call()
        same = True
        for _ in range(3):                     # replays interleaved with eager work, each checked
            h.zero_(); logits.zero_(); value.zero_()
            g.replay()
            torch.cuda.synchronize()
            same = same and bool(torch.equal(h, ref[0]) and torch.equal(logits, ref[1]) and torch.equal(value, ref[2]))
            call()
            torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(calls):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) / calls * 1e3
    except Exception as e:                      # capture is an extra; the eager figure stands on its own
        graph_ms, same = None, "capture failed: %s" % (str(e)[:120],)
    out = {"tokens": n_tokens, "calls": calls, "launch_per_kernel_ms_per_state": round(eager_ms, 4),
           "hip_graph_replay_ms_per_state": None if graph_ms is None else round(graph_ms, 4),
           "graph_replays_match_eager": same,
           "states_per_s_one_at_a_time": round(1e3 / (graph_ms if graph_ms else eager_ms), 1)}
    if graph_ms is not None:
        try:
            out["independent_agents"] = _concurrent_agents(torch, B, R, synth, np, enc, head, shape)
        except Exception as e:
            out["independent_agents"] = "failed: %s" % (str(e)[:120],)
    return out


def _concurrent_agents(torch, B, R, synth, np, enc, head, shape, n_agents: int = 8, rounds: int = 30):
    """n_agents independent callers, each with its own short state, buffers, stream (default priority) and captured
    graph of encoder_forward_packed + heads; every round replays all graphs, one per stream.  The library keeps no
    state between calls, so the replays may overlap on the GPU: one short state leaves most of it idle."""
    agents = []
    for a in range(n_agents):
        n = 15 + (a * 7) % 26                    # 15 .. 40 tokens
        ids = R.dev(synth.token_ids(0, 520 + a, (n,), shape.vocab))
        cu_host = np.asarray([0, n], dtype=np.int32)
        ag = {"n": n, "ids": ids, "cu_host": cu_host, "cu_dev": R.dev(cu_host),
              "ws": R.Workspace(B.brl_encoder_packed_workspace_bytes(enc.struct, 1, n, n)),
              "hws": R.Workspace(B.brl_head_workspace_bytes(head.struct, 1)),
              "h": torch.empty((1, shape.d), dtype=torch.float32, device="cuda"),
              "logits": torch.empty((1, head.n_actions), dtype=torch.float32, device="cuda"),
              "value": torch.empty((1,), dtype=torch.float32, device="cuda"),
              "stream": torch.cuda.Stream()}

        def call(ag=ag):
            B.encoder_forward_packed(enc.struct, ag["ids"], ag["cu_dev"], ag["cu_host"], 1, ag["n"], ag["h"], ag["ws"].buf)
            B.policy_value_head(head.struct, ag["h"], 1, ag["logits"], ag["value"], ag["hws"].buf)

        call()
        torch.cuda.synchronize()
        ag["ref"] = ag["h"].clone()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            call()
        ag["graph"] = g
        agents.append(ag)
    main = torch.cuda.current_stream()

    def one_round():
        for ag in agents:
            ag["stream"].wait_stream(main)
            with torch.cuda.stream(ag["stream"]):
                ag["graph"].replay()
        for ag in agents:
            main.wait_stream(ag["stream"])

    same = True
    for _ in range(3):
        for ag in agents:
            ag["h"].zero_()
        one_round()
        torch.cuda.synchronize()
        same = same and all(bool(torch.equal(ag["h"], ag["ref"])) for ag in agents)
    t0 = time.perf_counter()
    for _ in range(rounds):
        one_round()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / rounds * 1e3
    return {"agents": n_agents, "tokens_per_state": [ag["n"] for ag in agents], "ms_per_round": round(ms, 4),
            "states_per_s": round(n_agents / ms * 1e3, 1), "each_matches_its_own_call": same}


def bench_critics(torch, B, R, synth, enc, ids, Bn: int, S: int, shape, steps: int, warmup: int):
    """The hybrid-precision and ensemble rows of the paper's ablation table: the same batch through the int8-weight
    encoder (per-tensor absmax int8 weights of the same master matrices), and 1 / 3 / 5 value heads on the cached h."""
    twin = enc.int8_twin
    twin.ws = R.Workspace(B.brl_encoder_workspace_bytes(twin.struct, Bn, S))
    h8 = torch.empty((Bn, shape.d), dtype=torch.float32, device="cuda")

    def run():
        B.encoder_forward(twin.struct, ids, Bn, S, None, h8, twin.ws.buf)

    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    for k in range(len(B.KERNEL_CLASSES)):
        B.brl_timing_read(k)
    B.brl_timing_enable(True)
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    B.brl_timing_enable(False)
    n, gms, ops = B.brl_timing_read_ops(B.BRL_KC_GEMM_NARROW)
    for k in range(len(B.KERNEL_CLASSES)):
        B.brl_timing_read(k)
    h1 = enc.forward(ids)
    out = {"int8_weight_encoder": {"ms_per_step": round(ms, 4), "states_per_s": round(Bn / ms * 1e3, 1),
                                   "weight_bytes": int(sum(t[k].packed.numel() for t in enc.keep[1::2] for k in t
                                                           if hasattr(t[k], "packed"))),
                                   "gemm_kernel": "gemm_lds_w8_kernel<2,2,2,2>",
                                   "gemm_ms_per_step": round(gms / steps, 4),
                                   "gemm_tops": round(ops / (gms * 1e-3) / 1e12, 2) if gms > 0 else 0.0}}
    dims = [shape.d, 256, 1]
    ens = {}
    for n_members in (1, 3, 5):
        e = R.ValueEnsemble([synth.mlp_params(0, 400 + 20 * i, dims) for i in range(n_members)])
        for _ in range(5):
            e.forward(h1, want_each=False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(50):
            e.forward(h1, want_each=False)
        torch.cuda.synchronize()
        ens["%d_heads_us" % n_members] = round((time.perf_counter() - t0) / 50 * 1e6, 1)
    out["value_ensemble"] = dict(ens, batch=Bn, dims=dims, launches_per_call=3)
    return out


def bench_ppo(torch, B, R, synth, np, shape, want_cpu: bool, T: int = 2048, batch: int = 64, epochs: int = 4):
    """One PPO update of the 2560->256->{18,1} heads on a cached 2048-step rollout (mini-batches of 64, 4 epochs:
    128 optimiser steps), hyper-parameters of the paper's table; the oracle's fp64 update timed beside it."""
    dims_p, dims_v = [shape.d, 256, shape.n_actions], [shape.d, 256, 1]
    c = synth.ppo_rollout_case(0, T, shape.d, shape.n_actions, epochs)
    pw, pb = synth.mlp_params(0, 60, dims_p)
    vw, vb = synth.mlp_params(0, 80, dims_v)
    rew, val, don, last = R.dev(c["rewards"]), R.dev(c["values"]), R.dev(c["dones"]), R.dev(c["last_value"])
    h, actions, logp_old, perm = R.dev(c["h"]), R.dev(c["actions"]), R.dev(c["logp_old"]), R.dev(c["perm"])

    def run():
        tr = R.PPOTrainer((pw, pb), (vw, vb))
        adv, ret = R.gae(rew, val, don, last, 0.99, 0.95)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        tr.update(h, actions, logp_old, adv.reshape(-1), ret.reshape(-1), perm, batch, want_stats=False)
        torch.cuda.synchronize()
        return tr, (time.perf_counter() - t0) * 1e3

    run()
    times = []
    for _ in range(3):
        tr, ms = run()
        times.append(ms)
    ms = min(times)
    steps = epochs * (T // batch)
    out = {"rollout_steps": T, "batch": batch, "epochs": epochs, "optimiser_steps": steps, "ms_per_update": round(ms, 3),
           "us_per_optimiser_step": round(ms / steps * 1e3, 2), "trainable_params": int(tr.params.numel()),
           "kernel_launches_per_update": steps * 8, "cpu_oracle": None}
    if want_cpu:
        from oracle import ppo_oracle as P
        adv_ref, ret_ref = P.gae(c["rewards"][0], c["values"][0], c["dones"][0], c["last_value"][0], 0.99, 0.95)
        pol = P.MLPParams([w.astype(np.float64) for w in pw], [b.astype(np.float64) for b in pb])
        vl = P.MLPParams([w.astype(np.float64) for w in vw], [b.astype(np.float64) for b in vb])
        t0 = time.perf_counter()
        P.ppo_update(c["h"].astype(np.float64), c["actions"], c["logp_old"].astype(np.float64),
                     adv_ref.astype(np.float32).astype(np.float64), ret_ref.astype(np.float32).astype(np.float64),
                     pol, vl, c["perm"], batch, P.PPOHyper())
        cpu_ms = (time.perf_counter() - t0) * 1e3
        got = tr.tensors()
        dev_max = max(float(np.abs(g.astype(np.float64) - w).max()) for g, w in zip(got[0] + got[2], pol.weights + vl.weights))
        out["cpu_oracle"] = {"ms_per_update": round(cpu_ms, 1), "kind": "oracle (NumPy fp64)",
                             "max_abs_weight_difference_gpu_vs_oracle": dev_max}
    return out


def bench_gemv(torch, B, R, synth, calls: int, n_pairs: int = 256, n_drawn: int = 8):
    """Decode-shape pair x[1,2560] -> up[6912] -> down[2560]: streaming over a pool of weight-pair buffers (by
    default one pair per call: 8.8 GB, every weight byte is read once per batched launch and the 256 MB last-level
    cache cannot serve any of it), and resident on one pair.  The first n_drawn pairs are seeded Philox draws
    (synth.gemv_pair_case, ternarised and packed by the library); the rest of the pool are device copies of their
    packed blobs in buffers of their own: what a streaming kernel sees is addresses and bit statistics, and host
    draws of 1000 pairs (35 G normals) would take many minutes."""
    d, f = 2560, 6912
    from paper_2604_24273_amd.runtime import PackedLinear
    drawn = []
    for i in range(min(n_drawn, n_pairs)):
        c = synth.gemv_pair_case(0, d, f, pair=i)
        drawn.append((R.quantize_linear(c["W_up"]), R.quantize_linear(c["W_down"])))
    pairs = list(drawn)
    while len(pairs) < n_pairs:
        up, dn = drawn[len(pairs) % len(drawn)]
        pairs.append((PackedLinear(up.packed.clone(), up.beta.clone(), up.n_out, up.k_in),
                      PackedLinear(dn.packed.clone(), dn.beta.clone(), dn.n_out, dn.k_in)))
    x = R.dev(synth.normal(0, 10, (1, d)))
    h = torch.empty((1, f), dtype=torch.float32, device="cuda")
    y = torch.empty((1, d), dtype=torch.float32, device="cuda")
    ws = R.Workspace(max(B.brl_bitlinear_workspace_bytes(1, f, d), B.brl_bitlinear_workspace_bytes(1, d, f)))
    bytes_pair = 2 * B.brl_packed_bytes(f, d) + (d + f) + 4 * (d + f)     # packed W + int8 x + fp32 y

    def run(pool_size, n):
        for i in range(n):
            up, dn = pairs[i % pool_size]
            B.bitlinear_forward(up.packed, up.beta, f, d, x, 1, 1e-5, h, None, None, None, None, ws.buf)
            B.bitlinear_forward(dn.packed, dn.beta, d, f, h, 1, 1e-5, y, None, None, None, None, ws.buf)

    res = {"bytes_per_pair": bytes_pair, "calls": calls, "pool_pairs": n_pairs, "pool_pairs_drawn": len(drawn),
           "pool_bytes": n_pairs * 2 * B.brl_packed_bytes(f, d),
           "bytes_walked_per_batched_launch": min(calls, n_pairs) * B.brl_packed_bytes(f, d),
           "last_level_cache_bytes": 256 * 2 ** 20}
    for mode, pool_size in (("streaming", n_pairs), ("resident", 1)):
        run(pool_size, 50)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(pool_size, calls)
        torch.cuda.synchronize()
        wall_us = (time.perf_counter() - t0) / calls * 1e6
        B.brl_timing_enable(True)
        run(pool_size, calls)
        torch.cuda.synchronize()
        B.brl_timing_enable(False)
        n, ms = B.brl_timing_read(B.BRL_KC_GEMV)
        kern_us_pair = ms / max(n, 1) * 2 * 1e3
        gbs = bytes_pair / (kern_us_pair * 1e-6) / 1e9 if kern_us_pair > 0 else 0.0
        res[mode] = {"wall_us_per_pair": round(wall_us, 3), "kernel_us_per_pair": round(kern_us_pair, 3),
                     "kernel_GBps": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
                     "wall_GBps": round(bytes_pair / (wall_us * 1e-6) / 1e9, 1)}
    res["roofline_launch_per_call"] = {"bound": "hbm", "kernel": "gemv_kernel<1>",
                                       "achieved": res["streaming"]["kernel_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                       "frac": res["streaming"]["frac_of_hbm_peak"], "traffic": None}

    # The same `calls` pairs as two launches: every up product in one bitlinear_forward_batch, then every
    # down product on the h rows the first launch wrote (each pair keeps its own h and y).
    hs = torch.empty((calls, 1, f), dtype=torch.float32, device="cuda")
    ys = torch.empty((calls, 1, d), dtype=torch.float32, device="cuda")

    def ptrs(vals):
        return torch.tensor(vals, dtype=torch.int64, device="cuda")

    idx = [i % n_pairs for i in range(calls)]
    up_w, up_b = ptrs([pairs[i][0].packed.data_ptr() for i in idx]), ptrs([pairs[i][0].beta.data_ptr() for i in idx])
    dn_w, dn_b = ptrs([pairs[i][1].packed.data_ptr() for i in idx]), ptrs([pairs[i][1].beta.data_ptr() for i in idx])
    x_p = ptrs([x.data_ptr()] * calls)
    h_p = ptrs([hs[i].data_ptr() for i in range(calls)])
    y_p = ptrs([ys[i].data_ptr() for i in range(calls)])

    def run_batch():
        B.bitlinear_forward_batch(up_w, up_b, f, d, x_p, B.BRL_F32, 1, 1e-5, h_p, calls)
        B.bitlinear_forward_batch(dn_w, dn_b, d, f, h_p, B.BRL_F32, 1, 1e-5, y_p, calls)

    run_batch()
    torch.cuda.synchronize()
    same = bool(torch.equal(ys[0], y))        # pair 0: the resident launch-per-call leg ended on it
    reps = 5
    t0 = time.perf_counter()
    for _ in range(reps):
        run_batch()
    torch.cuda.synchronize()
    wall_us = (time.perf_counter() - t0) / (reps * calls) * 1e6
    B.brl_timing_enable(True)
    for _ in range(reps):
        run_batch()
    torch.cuda.synchronize()
    B.brl_timing_enable(False)
    n, ms = B.brl_timing_read(B.BRL_KC_GEMV)
    kern_us_pair = ms / (reps * calls) * 1e3
    gbs = bytes_pair / (kern_us_pair * 1e-6) / 1e9 if kern_us_pair > 0 else 0.0
    res["one_launch_batch"] = {"pairs_per_launch": calls, "launches": 2, "pair0_equals_launch_per_call_result": same,
                               "wall_us_per_pair": round(wall_us, 3),
                               "kernel_us_per_pair": round(kern_us_pair, 3), "kernel_GBps": round(gbs, 1),
                               "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
                               "wall_GBps": round(bytes_pair / (wall_us * 1e-6) / 1e9, 1)}
    res["roofline"] = {"bound": "hbm", "kernel": "gemv_batch_kernel<1> (all pairs of the pool walk in two launches)",
                       "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                       "frac": round(gbs / HBM_PEAK_GBS, 4),
                       "traffic": None if GEMV_BATCH_FETCH["ratio"] is None
                       else round(GEMV_BATCH_FETCH["ratio"] * calls * bytes_pair / 2),
                       "traffic_source": GEMV_BATCH_FETCH["source"]}
    return res


if __name__ == "__main__":
    sys.exit(main())
