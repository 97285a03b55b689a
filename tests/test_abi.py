"""Host-side checks that need no GPU: the library loads, exports every symbol the
header declares, answers its size queries and rejects bad arguments before any
kernel would be enqueued."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2604_24273_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2604_24273_amd import build
        build.build()
    binding.lib()
    return binding


def _declared_functions():
    src = open(os.path.join(ROOT, "include", "bitrl.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = re.findall(r"\b([a-z_][a-z0-9_]*)\s*\([^;{}]*\)\s*;", src)
    return sorted(set(names))


def test_header_symbols_are_exported_and_bound(B):
    names = _declared_functions()
    assert {"bitlinear_quantize_weights", "bitlinear_forward", "ffn_block_forward", "encoder_forward",
            "policy_value_head"} <= set(names)
    handle = B.lib()
    for n in names:
        assert hasattr(handle, n), n
    assert set(names) == set(B.EXPORTS)
    assert B.brl_abi_version() == 2


def test_struct_layouts_match_the_header(B):
    p = C.sizeof(C.c_void_p)
    assert C.sizeof(B.brl_ffn_weights) == 8 * p
    assert C.sizeof(B.brl_layer_weights) == 10 * p + 8 * p
    assert C.sizeof(B.brl_encoder) == 7 * 4 + 3 * 4 + 4 + 4 + 3 * p    # 7 ints, 3 floats, 1 int, pad, 3 pointers
    assert C.sizeof(B.brl_mlp) == 8 + 3 * p + 8


def test_size_queries(B):
    assert B.brl_packed_bytes(2048, 2048) == 2048 * 2048 // 4
    assert B.brl_packed_bytes(6912, 2560) == 4423680            # 2-bit packed decode-shape matrix
    assert B.brl_packed_bytes(70, 200) == 96 * 256 // 4          # rows pad to 32, columns to 128
    assert B.brl_packed_bytes(0, 5) == 0
    assert B.brl_bitlinear_workspace_bytes(1, 6912, 2560) > 0
    assert B.brl_bitlinear_workspace_bytes(256, 6912, 2560) >= 256 * 2560
    assert B.brl_ffn_workspace_bytes(256, 2560, 6912) >= 256 * 6912 * 4
    assert B.brl_quantize_workspace_bytes(10, 10) >= 8192


def test_bad_arguments_are_rejected_on_the_host(B):
    lib = B.lib()
    fake = C.c_void_p(0x1000)          # aligned, never dereferenced: checks fail first
    odd = C.c_void_p(0x1004)

    def err():
        return lib.brl_last_error().decode()

    # null / misaligned pointers
    assert lib.bitlinear_forward(None, fake, 32, 128, fake, 0, 1, 1e-5, fake, None, None, None, None, fake, 1 << 30, None) == B.BRL_EINVAL
    assert "null" in err()
    assert lib.bitlinear_forward(fake, fake, 32, 128, odd, 0, 1, 1e-5, fake, None, None, None, None, fake, 1 << 30, None) == B.BRL_EINVAL
    assert "aligned" in err()
    # shapes
    assert lib.bitlinear_forward(fake, fake, 32, 100, fake, 0, 1, 1e-5, fake, None, None, None, None, fake, 1 << 30, None) == B.BRL_EINVAL
    assert "multiple of 8" in err()
    assert lib.bitlinear_forward(fake, fake, 32, 16384, fake, 0, 1, 1e-5, fake, None, None, None, None, fake, 1 << 30, None) == B.BRL_EINVAL
    assert lib.bitlinear_forward(fake, fake, 32, 128, fake, 0, 0, 1e-5, fake, None, None, None, None, fake, 1 << 30, None) == B.BRL_EINVAL
    assert lib.bitlinear_forward(fake, fake, 32, 128, fake, 7, 1, 1e-5, fake, None, None, None, None, fake, 1 << 30, None) == B.BRL_EINVAL
    # the batch entry point: few-token problems only, sane counts and shapes
    assert lib.bitlinear_forward_batch(None, fake, 32, 128, fake, 0, 1, 1e-5, fake, 1, None) == B.BRL_EINVAL
    assert lib.bitlinear_forward_batch(fake, fake, 32, 128, fake, 0, 5, 1e-5, fake, 1, None) == B.BRL_EINVAL
    assert lib.bitlinear_forward_batch(fake, fake, 32, 128, fake, 0, 0, 1e-5, fake, 1, None) == B.BRL_EINVAL
    assert lib.bitlinear_forward_batch(fake, fake, 32, 128, fake, 0, 1, 1e-5, fake, -1, None) == B.BRL_EINVAL
    assert lib.bitlinear_forward_batch(fake, fake, 32, 100, fake, 0, 1, 1e-5, fake, 1, None) == B.BRL_EINVAL
    assert lib.bitlinear_forward_batch(fake, fake, 32, 128, fake, 9, 1, 1e-5, fake, 1, None) == B.BRL_EINVAL
    # workspace too small
    assert lib.bitlinear_forward(fake, fake, 32, 128, fake, 0, 64, 1e-5, fake, None, None, None, None, fake, 16, None) == B.BRL_ENOSPC
    assert "workspace" in err()
    assert lib.bitlinear_quantize_weights(fake, 4, 4, 1e-5, fake, fake, None, fake, 8, None) == B.BRL_ENOSPC
    assert lib.bitlinear_quantize_weights(fake, 0, 4, 1e-5, fake, fake, None, fake, 1 << 20, None) == B.BRL_EINVAL
    # ffn / encoder / head tables
    w = B.brl_ffn_weights()
    assert lib.ffn_block_forward(C.byref(w), fake, 0, 4, 128, 256, 1e-5, 1e-5, fake, fake, 1 << 30, None) == B.BRL_EINVAL
    enc = B.brl_encoder()
    assert lib.encoder_forward(C.byref(enc), fake, 1, 1, None, fake, fake, 1 << 30, None) == B.BRL_EINVAL
    enc = B.brl_encoder(0, 256, 4, 3, 64, 512, 100, 1e4, 1e-5, 1e-5, 0, 0, 0x1000, 0x1000, None)
    assert lib.encoder_forward(C.byref(enc), fake, 1, 1, None, fake, fake, 1 << 30, None) == B.BRL_EINVAL
    assert "n_kv_heads" in err()
    enc = B.brl_encoder(0, 256, 4, 2, 48, 512, 100, 1e4, 1e-5, 1e-5, 0, 0, 0x1000, 0x1000, None)
    assert lib.encoder_forward(C.byref(enc), fake, 1, 1, None, fake, fake, 1 << 30, None) == B.BRL_EINVAL
    assert "head_dim" in err()
    # PPO head update: shapes and hyper-parameters are checked on the host
    cfg, keep = B.make_ppo_config([16, 8, 4], [16, 8, 1], B.BRL_ACT_TANH)
    assert lib.brl_ppo_param_count(C.byref(cfg)) == 16 * 8 + 8 + 8 * 4 + 4 + 16 * 8 + 8 + 8 + 1
    w_off, b_off = B.brl_ppo_param_offsets(cfg)
    assert w_off == [0, 136, 172, 308] and b_off == [128, 168, 300, 316]
    assert lib.brl_ppo_workspace_bytes(C.byref(cfg), 64) > 0
    step = C.c_longlong(0)
    args = (fake,) * 3 + (C.byref(step),) + (fake,) * 5
    assert lib.ppo_head_update(C.byref(cfg), *args, 128, fake, 1, 64, None, fake, 16, None) == B.BRL_ENOSPC
    assert lib.ppo_head_update(C.byref(cfg), *args, 128, fake, 1, 256, None, fake, 1 << 30, None) == B.BRL_EINVAL   # batch > T
    assert lib.ppo_head_update(C.byref(cfg), *args, 128, fake, 1, 1, None, fake, 1 << 30, None) == B.BRL_EINVAL     # normalisation of one sample
    assert lib.ppo_head_update(C.byref(cfg), *args, 128, None, 1, 64, None, fake, 1 << 30, None) == B.BRL_EINVAL
    bad, keep2 = B.make_ppo_config([16, 8, 4], [12, 8, 1], B.BRL_ACT_TANH)
    assert lib.brl_ppo_param_count(C.byref(bad)) == 0 and "input width" in err()
    bad, keep3 = B.make_ppo_config([16, 8, 4], [16, 8, 2], B.BRL_ACT_TANH)
    assert lib.brl_ppo_param_count(C.byref(bad)) == 0 and "one output" in err()
    assert lib.ppo_gae(fake, fake, fake, fake, 1, 0, 0.99, 0.95, fake, fake, None) == B.BRL_EINVAL
    assert lib.ppo_gae(fake, fake, fake, fake, 1, 8, 1.5, 0.95, fake, fake, None) == B.BRL_EINVAL
    # packed layout: the host copy of the cumulative lengths is checked before anything is launched
    enc = B.brl_encoder(0, 256, 4, 2, 64, 512, 100, 1e4, 1e-5, 1e-5, 0, 0, 0x1000, 0x1000, None)
    import numpy as np
    for cu, max_len in (([1, 5], 8), ([0, 5, 5], 8), ([0, 9], 8), ([0, 3, 2], 8)):
        cu_h = np.asarray(cu, dtype=np.int32)
        rc = lib.encoder_forward_packed(C.byref(enc), fake, fake, cu_h.ctypes.data, len(cu) - 1, max_len, fake, fake,
                                        1 << 30, None)
        assert rc == B.BRL_EINVAL, cu
    cu_h = np.asarray([0, 3, 8], dtype=np.int32)
    assert lib.encoder_forward_packed(C.byref(enc), fake, fake, cu_h.ctypes.data, 2, 8, fake, fake, 16, None) == B.BRL_ENOSPC
    assert lib.brl_encoder_packed_workspace_bytes(C.byref(enc), 2, 8, 8) > 0
    assert lib.brl_encoder_packed_workspace_bytes(C.byref(enc), 2, 1, 8) == 0
    head = B.brl_head()
    assert lib.policy_value_head(C.byref(head), fake, 1, fake, fake, fake, 1 << 20, None) == B.BRL_EINVAL
    # int8-weight variant and ensemble critic
    enc = B.brl_encoder(0, 256, 4, 2, 64, 512, 100, 1e4, 1e-5, 1e-5, 0, 7, 0x1000, 0x1000, None)
    assert lib.encoder_forward(C.byref(enc), fake, 1, 1, None, fake, fake, 1 << 30, None) == B.BRL_EINVAL
    assert "weight_format" in err()
    assert lib.brl_packed_int8_bytes(33, 130) == 64 * 256 and lib.brl_packed_int8_bytes(0, 8) == 0
    assert lib.bitlinear_quantize_weights_int8(fake, 4, 4, 0.0, 127, fake, fake, None, fake, 1 << 20, None) == B.BRL_EINVAL
    assert lib.bitlinear_quantize_weights_int8(fake, 4, 4, 1e-5, 127, fake, fake, None, fake, 8, None) == B.BRL_ENOSPC
    assert lib.bitlinear_quantize_weights_int8(fake, 4, 4, 1e-5, 128, fake, fake, None, fake, 1 << 20, None) == B.BRL_EINVAL
    assert "qmax" in err()
    assert lib.bitlinear_int8_forward(fake, fake, 32, 100, fake, 0, 1, 1e-5, fake, None, None, None, None, fake, 1 << 20, None) == B.BRL_EINVAL
    assert lib.bitlinear_int8_forward(fake, fake, 32, 128, fake, 0, 64, 1e-5, fake, None, None, None, None, fake, 16, None) == B.BRL_ENOSPC
    import ctypes
    dims_a = (ctypes.c_int * 3)(16, 8, 1)
    dims_b = (ctypes.c_int * 3)(16, 4, 1)
    tbl = (ctypes.c_void_p * 2)(0x1000, 0x1000)
    mk = lambda dims: B.brl_mlp(2, ctypes.cast(dims, ctypes.POINTER(ctypes.c_int)), ctypes.cast(tbl, ctypes.POINTER(ctypes.c_void_p)),
                                ctypes.cast(tbl, ctypes.POINTER(ctypes.c_void_p)), B.BRL_ACT_TANH)
    same = B.make_mlp_array([mk(dims_a), mk(dims_a), mk(dims_a)])
    assert lib.brl_value_ensemble_workspace_bytes(same, 3, 10) > 0
    assert lib.brl_value_ensemble_workspace_bytes(same, 9, 10) == 0
    assert lib.value_ensemble_forward(same, 3, fake, 10, fake, None, fake, 16, None) == B.BRL_ENOSPC
    assert lib.value_ensemble_forward(same, 0, fake, 10, fake, None, fake, 1 << 20, None) == B.BRL_EINVAL
    mixed = B.make_mlp_array([mk(dims_a), mk(dims_b)])
    assert lib.value_ensemble_forward(mixed, 2, fake, 10, fake, None, fake, 1 << 20, None) == B.BRL_EINVAL
    assert "differs" in err()


def test_product_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2604_24273_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith(".py"):
                txt = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in txt.replace("CPU oracle's tests", ""), fn


def test_profile_summary_reads_rocprof_csv(tmp_path):
    """The summariser behind profiles/*.txt: per-kernel averages from a kernel trace and a counter file."""
    from paper_2604_24273_amd import profile_summary as PS
    d = tmp_path / "out" / "host"
    d.mkdir(parents=True)
    (d / "1_kernel_trace.csv").write_text(
        '"Kind","Agent_Id","Queue_Id","Kernel_Id","Kernel_Name","Correlation_Id","Start_Timestamp","End_Timestamp"\n'
        '"KERNEL_DISPATCH",1,1,1,"k_a",1,1000,3000\n"KERNEL_DISPATCH",1,1,1,"k_a",2,5000,9000\n'
        '"KERNEL_DISPATCH",1,1,2,"k_b",3,100,200\n')
    (d / "1_counter_collection.csv").write_text(
        '"Dispatch_Id","Kernel_Name","Counter_Name","Counter_Value"\n1,"k_a","FETCH_SIZE",10\n2,"k_a","FETCH_SIZE",30\n')
    text = PS.summarise(str(tmp_path / "out"))
    row_a = [l for l in text.splitlines() if l.startswith("k_a") and "FETCH" not in l][0].split()
    assert row_a[1] == "2" and abs(float(row_a[2]) - 3.0) < 1e-9          # two calls, 3.00 us on average
    assert "avg 20" in [l for l in text.splitlines() if "FETCH_SIZE" in l][0]
