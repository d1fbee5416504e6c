"""The C-ABI library loads, exports every symbol include/based.h declares, and rejects bad
arguments on the host before anything is launched (no GPU needed: no compute call is made)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "based.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(based_[a-z_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def based():
    from paper_2402_18668_amd import based as b
    return b


def test_header_symbols_exported(based):
    names = declared_symbols()
    assert len(names) >= 14
    for n in names:
        assert hasattr(based.lib, n), n
    assert sorted(based.EXPORTS) == names


def test_size_queries(based):
    assert based.feature_dim(16) == 273 and based.feature_dim(32) == 1057 and based.feature_dim(0) == 0
    stride = based.state_stride_floats(16, 64)
    assert stride % 64 == 0 and stride >= 273 * 65
    assert based.state_bytes(2, 3, 16, 64) == 6 * stride * 4
    assert based.state_bytes(2, 3, 17, 64) == 0 and based.state_bytes(0, 3, 16, 64) == 0
    assert based.swa_ring_bytes(2, 3, 64, 128, based.BF16) == 6 * 2 * 64 * 128 * 2
    assert based.swa_ring_bytes(2, 3, 64, 128, based.F32) == 6 * 2 * 64 * 128 * 4
    assert based.swa_ring_bytes(2, 3, 48, 128, based.BF16) == 0
    assert based.prefill_workspace_bytes(1, 1, 100, 16, 64, based.F32) >= 0
    assert based.lib.based_version() >= 100
    # packed state: the paper's own state-size count (one row per unordered feature pair)
    assert based.lib.based_packed_feature_dim(16) == 153 and based.lib.based_packed_feature_dim(32) == 561
    assert based.lib.based_packed_feature_dim(0) == 0
    pstride = based.lib.based_packed_state_stride_floats(16, 128)
    assert pstride % 64 == 0 and pstride >= 153 * 129
    assert based.packed_state_bytes(2, 3, 16, 128) == 6 * pstride * 4
    assert based.packed_state_bytes(2, 3, 16, 100) == 0
    assert based.strerror(0) == "ok" and "unknown" in based.strerror(77)


def test_bad_arguments_are_rejected_before_launch(based):
    lib = based.lib
    p = ctypes.c_void_p(0x1000)      # aligned, never dereferenced: every call below fails validation
    odd = ctypes.c_void_p(0x1004)
    null = ctypes.c_void_p(0)
    st = ctypes.c_void_p(0)
    # prefill
    assert lib.based_prefill(null, p, p, p, null, 0, null, 1, 1, 8, 16, 64, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_prefill(odd, p, p, p, null, 0, null, 1, 1, 8, 16, 64, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_prefill(p, p, p, p, null, 0, null, 0, 1, 8, 16, 64, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_prefill(p, p, p, p, null, 0, null, 1, 1, -3, 16, 64, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_prefill(p, p, p, p, null, 1, null, 1, 1, 8, 16, 64, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_prefill(p, p, p, p, null, 0, null, 1, 1, 8, 20, 64, 1, st) == based.ERR_UNSUPPORTED
    assert lib.based_prefill(p, p, p, p, null, 0, null, 1, 1, 8, 16, 96, 1, st) == based.ERR_UNSUPPORTED
    assert lib.based_prefill(p, p, p, p, null, 0, null, 1, 1, 8, 16, 64, 7, st) == based.ERR_UNSUPPORTED
    assert lib.based_prefill(p, p, p, p, null, 0, null, 65536, 65536, 8, 16, 64, 1, st) == based.ERR_INVALID_ARG
    # status query: argument checks come before any device access; no waits in the fp32 / d' = 32 paths
    assert lib.based_prefill_status(odd, 1, 1, 8, 16, 64, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_prefill_status(p, 0, 1, 8, 16, 64, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_prefill_status(p, 1, 1, 8, 20, 64, 1, st) == based.ERR_UNSUPPORTED
    assert lib.based_prefill_status(null, 1, 1, 8, 16, 64, 0, st) == based.OK
    assert lib.based_prefill_status(null, 1, 1, 8, 32, 64, 1, st) == based.OK
    # the entry point on the library's static scratch: same host checks, and its size limit
    assert lib.based_prefill_static(null, p, p, p, null, 0, 1, 1, 8, 16, 64, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_prefill_static(p, p, p, p, null, 0, 1, 1, 8, 16, 96, 1, st) == based.ERR_UNSUPPORTED
    assert lib.based_prefill_static(p, p, p, p, null, 0, 64, 16, 8192, 32, 128, 1, st) == based.ERR_TOO_LARGE
    assert lib.based_prefill_status(null, 64, 16, 8192, 16, 128, 1, st) == based.ERR_TOO_LARGE
    lib.based_debug_set_poll_limit(5)
    lib.based_debug_set_poll_limit(-1)
    # decode
    assert lib.based_decode_step(p, p, p, p, null, 1, 1, 16, 64, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_decode_step(p, p, p, p, p, 1, 1, 16, 32, 1, st) == based.ERR_UNSUPPORTED
    # window attention
    assert lib.based_swa_prefill(p, p, null, p, null, 1, 1, 8, 64, 64, 0.125, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_swa_prefill(p, p, p, p, null, 1, 1, 8, 64, 48, 0.125, 1, st) == based.ERR_UNSUPPORTED
    assert lib.based_swa_decode(p, p, p, p, p, 0, 1, 1, 64, 64, 0.125, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_swa_decode(p, p, p, p, null, 1, 1, 1, 64, 64, 0.125, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_swa_decode(p, p, p, p, p, 1, 1, 1, 80, 64, 0.125, 1, st) == based.ERR_UNSUPPORTED
    # fused
    assert lib.based_decode_fused(p, p, p, p, p, 16, 64, p, p, p, p, p, 0, 64, 64, 0.125, 1, 1, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_decode_fused(p, p, p, p, p, 16, 64, p, p, p, p, null, 1, 64, 64, 0.125, 1, 1, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_decode_fused(p, p, p, p, p, 8, 64, p, p, p, p, p, 1, 64, 64, 0.125, 1, 1, 1, st) == based.ERR_UNSUPPORTED
    # packed-state variant
    assert lib.based_decode_step_packed(p, p, p, p, null, 1, 1, 16, 64, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_decode_step_packed(p, p, p, p, p, 1, 1, 16, 32, 1, st) == based.ERR_UNSUPPORTED
    assert lib.based_decode_fused_packed(p, p, p, p, p, 16, 64, p, p, p, p, p, 0, 64, 64, 0.125, 1, 1, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_prefill_packed(p, p, p, p, null, 0, null, 1, 1, 8, 16, 64, 0, st) == based.ERR_UNSUPPORTED   # fp32
    assert lib.based_prefill_packed(p, p, p, p, null, 1, p, 1, 1, 8, 16, 64, 1, st) == based.ERR_INVALID_ARG     # no state
    assert lib.based_prefill_packed(p, p, p, p, p, 0, null, 1, 1, 8, 32, 64, 1, st) == based.ERR_INVALID_ARG     # no workspace
    assert lib.based_state_pack(p, null, 1, 1, 16, 64, st) == based.ERR_INVALID_ARG
    assert lib.based_state_unpack(p, p, 1, 1, 12, 64, st) == based.ERR_UNSUPPORTED
    # projection
    assert lib.based_linear(null, p, p, 8, 64, 128, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_linear(p, p, p, 0, 64, 128, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_linear(p, p, p, 8, 48, 128, 1, st) == based.ERR_UNSUPPORTED
    assert lib.based_linear(p, p, p, 8, 64, 100, 1, st) == based.ERR_UNSUPPORTED
    assert lib.based_linear(p, p, p, 8, 64, 128, 0, st) == based.ERR_UNSUPPORTED
    # head-major projections
    assert lib.based_project_qkv(null, p, p, p, p, 1, 8, 64, 8, 16, 64, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_project_qkv(p, p, p, p, p, 1, 8, 64, 8, 16, 64, 0, st) == based.ERR_UNSUPPORTED
    assert lib.based_project_qkv(p, p, p, p, p, 1, 8, 64, 3, 16, 64, 1, st) == based.ERR_UNSUPPORTED
    assert lib.based_project_out(p, p, null, 1, 8, 8, 64, 128, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_project_out(p, p, p, 1, 8, 8, 32, 128, 1, st) == based.ERR_UNSUPPORTED
    # rotary
    assert lib.based_rotary_table(null, 0, 4, 64, 10000.0, st) == based.ERR_INVALID_ARG
    assert lib.based_rotary_table(p, -1, 4, 64, 10000.0, st) == based.ERR_INVALID_ARG
    assert lib.based_rotary_table(p, 0, 4, 64, 1.0, st) == based.ERR_INVALID_ARG
    assert lib.based_rotary_table(p, 0, 4, 80, 10000.0, st) == based.ERR_UNSUPPORTED
    assert lib.based_swa_prefill_rotary(p, p, p, p, null, null, 1, 1, 8, 64, 64, 0.125, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_swa_prefill_rotary(p, p, p, p, null, p, 1, 1, 8, 64, 48, 0.125, 1, st) == based.ERR_UNSUPPORTED
    assert lib.based_swa_decode_rotary(p, p, p, p, p, p, 4, 5, null, 1, 1, 64, 64, 0.125, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_swa_decode_rotary(p, p, p, p, p, null, 4, 1, null, 1, 1, 64, 64, 0.125, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_swa_decode_rotary(p, p, p, p, p, p, 4, 0, null, 1, 1, 64, 64, 0.125, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_decode_fused_rotary(p, p, p, p, p, 0, 16, 64, p, p, p, p, p, null, 4, 1, null, 64, 64, 0.125, 1, 1, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_decode_fused_rotary(p, p, p, p, p, 0, 16, 64, p, p, p, p, p, p, 4, 5, null, 64, 64, 0.125, 1, 1, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_decode_fused_rotary(p, p, p, p, p, 0, 8, 64, p, p, p, p, p, p, 4, 1, null, 64, 64, 0.125, 1, 1, 1, st) == based.ERR_UNSUPPORTED
    # decay variant
    assert lib.based_prefill_decay(p, p, p, p, null, 0, null, null, null, 1, 1, 8, 16, 64, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_prefill_decay(p, p, p, p, null, 0, null, p, null, 1, 1, 8, 20, 64, 1, st) == based.ERR_UNSUPPORTED
    assert lib.based_decode_step_decay(p, p, p, p, p, null, null, 1, 1, 16, 64, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_prefill_decay_workspace_bytes(1, 1, 8, 16, 64, 1) == 0
    assert lib.based_prefill_decay_workspace_bytes(1, 2, 4096, 16, 64, 1) > 0
    # BaseConv gate
    assert lib.based_short_conv_gate(null, p, p, p, p, null, p, null, 1, 4, 64, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_short_conv_gate(p, p, p, p, p, null, p, null, 1, 0, 64, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_short_conv_gate(p, p, p, p, p, null, p, null, 1, 4, 60, 1, st) == based.ERR_UNSUPPORTED
    assert lib.based_short_conv_gate(p, p, p, p, p, p, p, p, 1, 33, 64, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_short_conv_gate(p, p, p, p, p, odd, p, null, 1, 4, 64, 1, st) == based.ERR_INVALID_ARG
    # numerator-only variants validate like the calls they mirror
    assert lib.based_prefill_numerator(null, p, p, p, null, 0, null, 1, 1, 8, 16, 64, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_prefill_numerator(p, p, p, p, null, 0, null, 1, 1, 8, 20, 64, 1, st) == based.ERR_UNSUPPORTED
    assert lib.based_decode_step_numerator(p, p, p, p, null, 1, 1, 16, 64, 1, st) == based.ERR_INVALID_ARG
    assert lib.based_decode_step_numerator(p, p, p, p, p, 1, 1, 12, 64, 1, st) == based.ERR_UNSUPPORTED
    # position bookkeeping
    assert lib.based_positions_advance(null, 4, st) == based.ERR_INVALID_ARG
    assert lib.based_positions_advance(p, 0, st) == based.ERR_INVALID_ARG
    # d' = 32 in bf16 always needs the workspace
    assert lib.based_prefill(p, p, p, p, null, 0, null, 1, 1, 8, 32, 64, 1, st) == based.ERR_INVALID_ARG
    # state copies
    assert lib.based_state_export(null, p, p, 1, 1, 16, 64, st) == based.ERR_INVALID_ARG
    assert lib.based_state_import(p, p, p, 1, 1, 16, 100, st) == based.ERR_UNSUPPORTED


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU only: --gpus 2 exits with a message and a non-zero status before
    touching any device; the credited-work helper matches the hand count for both state layouts."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_mod", os.path.join(root, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    # 4 D d_v + 4 D + (C + 1)(d' + d_v + 1) with D = 273 (unpacked) and 153 (one row per unordered pair)
    assert mod.lin_prefill_flops_per_token_head(16, 64, packed=False) == 4 * 273 * 64 + 4 * 273 + 65 * 81
    assert mod.lin_prefill_flops_per_token_head(16, 64, packed=True) == 4 * 153 * 64 + 4 * 153 + 65 * 81 == 45045
