"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every declared symbol, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2604_12247_amd as sb
from paper_2604_12247_amd import binding as B
import sb_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "specbound.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(sb_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(sb.SYMBOLS), declared ^ set(sb.SYMBOLS)
    L = sb.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_struct_layouts_match_header_sizes():
    assert C.sizeof(B.sb_config) == 16 * 4
    assert C.sizeof(B.sb_draft_result) == 16
    assert C.sizeof(B.sb_verify_result) == (5 + 2 * sb.SB_MAX_W) * 4
    assert C.sizeof(B.sb_stats) == 8 * 8 + 9 * 8 + 65 * 8 + 2 * 8 + 2 * 8 + 7 * 8 + 3 * 8


def test_temperature_schedule_eq1(golden):
    gd = golden("paper_equations.txt")
    T = sb.temperature_schedule(gd["eq1_alpha"][0], gd["eq1_L"][0], gd["eq1_L"][0])
    for l, want in zip(gd["eq1_layers"], gd["eq1_T"]):
        assert abs(float(T[l - 1]) - want) < 1e-6
    assert float(T[-1]) == 1.0


def test_rope_table_host_values():
    c, s = sb.rope_table(4, 10000.0, 60)
    assert c.shape == (60, 2)
    assert np.all(c[0] == 1.0) and np.all(s[0] == 0.0)
    assert abs(c[50, 1] - np.cos(0.5)) < 1e-7 and abs(s[50, 1] - np.sin(0.5)) < 1e-7
    assert abs(c[3, 0] - np.cos(3.0)) < 1e-7


def test_query_sizes_and_config_validation():
    shape = si.CONFIGS["C2"].shape
    cfg = sb.make_config(shape, 1040)
    kv, ws = sb.query_sizes(cfg)
    assert kv == 32 * 2 * 1040 * 32 * 128 * 2
    assert ws > 8 * 4096 * 4
    bad = [dict(max_seq=1000), dict(head_dim=96), dict(n_kv_heads=5), dict(weight_dtype=7),
           dict(n_exit_heads=99), dict(d_model=4100), dict(vocab=0), dict(proj_kernel=9),
           dict(max_seq=65536 + 16),                       # more than 512 chunks of 128 keys
           dict(max_seq=32768 + 16, kv_dtype=sb.FP32)]     # an fp32 cache at head_dim 128 has 64-key chunks
    for kw in bad:
        cfg = sb.make_config(shape, 1040)
        for k, v in kw.items():
            setattr(cfg, k, v)
        with pytest.raises(sb.SbError) as e:
            sb.query_sizes(cfg)
        assert e.value.code == sb.EINVAL, kw
    cfg = sb.make_config(shape, 65536)                     # the longest context is accepted
    assert sb.query_sizes(cfg)[0] == 32 * 2 * 65536 * 32 * 128 * 2
    # the MFMA path is refused for fp32 weights
    cfg = sb.make_config(si.CONFIGS["C1"].shape, 112, sb.PROJ_MFMA)
    with pytest.raises(sb.SbError):
        sb.query_sizes(cfg)


def test_null_and_invalid_arguments_are_rejected_on_the_host():
    L = sb.lib()
    cfg = sb.make_config(si.CONFIGS["C1"].shape, 112)
    out = C.c_void_p()
    assert L.sb_load_model(C.byref(cfg), None, None, C.byref(out)) == sb.EINVAL
    assert b"NULL" in L.sb_last_error()
    w = B.sb_weights()          # all NULL pointers
    assert L.sb_load_model(C.byref(cfg), C.byref(w), None, C.byref(out)) == sb.EINVAL
    assert L.sb_new_session(None, None, 0, None, 0, None, C.byref(out)) == sb.EINVAL
    assert L.sb_prefill(None, None, 0, None) == sb.EINVAL
    assert L.sb_draft_step(None, None, None) == sb.EINVAL
    assert L.sb_verify(None, None, None) == sb.EINVAL
    assert L.sb_generate(None, None, 0, 0, None, None, 0, None, None) == sb.EINVAL
    assert L.sb_op_gemv(None, 0, 16, 64, None, None, 1, sb.PROJ_VALU, None, None) == sb.EINVAL
    x = np.zeros(64, np.float32)
    # shape rules of the single-kernel calls are checked before any launch
    assert L.sb_op_gemv(x.ctypes.data, 0, 16, 60, x.ctypes.data, x.ctypes.data, 1, sb.PROJ_VALU, None, None) == sb.EINVAL
    assert L.sb_op_gemv(x.ctypes.data, 0, 16, 64, x.ctypes.data, x.ctypes.data, 9, sb.PROJ_VALU, None, None) == sb.EINVAL
    assert L.sb_op_gemv(x.ctypes.data, 0, 16, 128, x.ctypes.data, x.ctypes.data, 1, sb.PROJ_MFMA, None, None) == sb.EINVAL
    assert L.sb_op_attention(x.ctypes.data, 4, 4, 64, 0, x.ctypes.data, x.ctypes.data, 2, 0, x.ctypes.data,
                             x.ctypes.data, 30, 4, x.ctypes.data, x.ctypes.data, None) == sb.ECAPACITY
    # the newer entry points reject NULL handles and bad shapes the same way
    assert L.sb_decode(None, 1, None, None, 0, None, None) == sb.EINVAL
    assert L.sb_rewind(None, 0, 0, 0) == sb.EINVAL
    assert L.sb_profile_begin(None, 0, 0, 1) == sb.EINVAL
    assert L.sb_profile_end(None, None, None, None, None) == sb.EINVAL
    assert L.sb_op_repack(None, 16, 128, None, None) == sb.EINVAL
    assert L.sb_op_repack(x.ctypes.data, 24, 128, x.ctypes.data, None) == sb.EINVAL     # N % 16
    assert L.sb_op_gemm(None, 16, 128, None, None, 1, None, None) == sb.EINVAL
    p = x.ctypes.data
    assert L.sb_op_gemm(p, 16, 128, p, p, 129, p, None) == sb.EINVAL                    # more than 128 rows
    assert L.sb_op_gemm(p, 16, 64, p, p, 1, p, None) == sb.EINVAL                       # K % 128
    assert L.sb_op_gemm(p, 20, 128, p, p, 1, p, None) == sb.EINVAL                      # N % 16
    assert L.sb_op_gemm_scratch_bytes(20, 128) == 0
    assert L.sb_op_prompt_attention(p, 4, 4, 64, p, p, 2, 0, p, p, 0, 33, p, None) == sb.ECAPACITY   # 33 rows, 2 pages
    assert L.sb_op_prompt_attention(p, 4, 4, 32, p, p, 2, 0, p, p, 0, 4, p, None) == sb.EINVAL       # head_dim
    assert L.sb_op_prompt_attention(p, 4, 4, 64, p, p, 2, 0, p, p, 0, 4, None, None) == sb.EINVAL
    assert L.sb_op_gemm_scratch_bytes(4096, 4096) >= 2 * 128 * 4096 * 2 + 128 * 4096 * 4


def test_new_config_fields_and_sizes_are_validated_on_the_host():
    L = sb.lib()
    shape = si.CONFIGS["C2"].shape
    cfg = sb.make_config(shape, 1040)
    out = B.sb_sizes()
    assert L.sb_query_sizes(C.byref(cfg), C.byref(out)) == 0
    # every projection matrix once more, tile-packed (each a multiple of 256 bytes here)
    es = 2
    per_layer = es * (shape.qkv_rows * shape.d_model + shape.d_model * shape.n_heads * shape.head_dim
                      + 3 * shape.d_ffn * shape.d_model)
    assert out.packed_weight_bytes == shape.n_layers * per_layer + (shape.n_exit_heads + 1) * es * shape.vocab * shape.d_model
    c1 = sb.make_config(si.CONFIGS["C1"].shape, 112)      # fp32 weights: no packed copy
    assert sb.packed_weight_bytes(c1) == 0
    for kw in (dict(kv_block=32), dict(max_w=9), dict(max_w=-1)):
        cfg = sb.make_config(shape, 1040)
        for k, v in kw.items():
            setattr(cfg, k, v)
        assert L.sb_query_sizes(C.byref(cfg), C.byref(out)) == sb.EINVAL, kw
    cfg = sb.make_config(shape, 1040)
    cfg.kv_block, cfg.max_w = 0, 0                         # defaults
    assert L.sb_query_sizes(C.byref(cfg), C.byref(out)) == 0
    # a packed-weight buffer that is misaligned or too small is refused before any device call
    w = B.sb_weights()
    dummy = np.zeros(64, np.float32)
    ptr = dummy.ctypes.data
    arr = (C.c_void_p * 32)(*([ptr] * 32))
    pa = C.cast(arr, C.POINTER(C.c_void_p))
    for name in ("embed", "final_norm", "lm_head"):
        setattr(w, name, ptr)
    for name in ("attn_norm", "w_qkv", "w_o", "ffn_norm", "w_gate_up", "w_down", "exit_norm", "exit_head"):
        setattr(w, name, pa)
    h = C.c_void_p()
    w.packed, w.packed_bytes = 4096 + 8, 1 << 40
    assert L.sb_load_model(C.byref(cfg), C.byref(w), None, C.byref(h)) == sb.EINVAL
    w.packed, w.packed_bytes = 4096, 1024
    assert L.sb_load_model(C.byref(cfg), C.byref(w), None, C.byref(h)) == sb.ENOMEM
    assert L.sb_debug_fail_launch(None, 1) == sb.EINVAL and L.sb_open_rows(None) == sb.EINVAL
    assert L.sb_phase_timing(None, 1) == sb.EINVAL
    x = np.zeros(64, np.float32).ctypes.data
    assert L.sb_op_head_static(x, 0, 131072 + 16, 64, x, 1, 1.0, sb.PROJ_VALU, x, x, None) == sb.ECAPACITY
