"""Host-only checks of the C ABI: the library loads, exports what include/dlm.h declares, and rejects bad arguments
before touching the GPU (no compute call is made here)."""
import ctypes as C
import os
import re

import pytest

from paper_2604_15750_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "dlm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dlm_\w+|block_boundary|select_parallel)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    L = api.lib()
    names = _declared()
    assert {"dlm_step", "block_boundary", "select_parallel", "dlm_model_create", "dlm_state_create"} <= set(names)
    for n in names:
        assert hasattr(L, n), n
    assert sorted(api.EXPORTS) == names


def test_struct_layouts_match_header():
    assert C.sizeof(api.dlm_config) == 11 * 4
    assert C.sizeof(api.dlm_weights) == 9 * 8
    assert C.sizeof(api.dlm_step_desc) == 8 + 18 * 8
    assert C.sizeof(api.dlm_boundary_params) == 20 and C.sizeof(api.dlm_select_params) == 16


def _err():
    return api.lib().dlm_last_error().decode()


def test_block_boundary_argument_errors():
    L = api.lib()
    one = C.c_void_p(16)  # never dereferenced: validation fails first
    p = api.dlm_boundary_params(1.2, 8, 1, 0, 0)
    z = (C.c_int32 * 1)(0)
    off = (C.c_int32 * 1)(4)
    call = lambda I=one, H=one, o=off, n=1, pp=p, Lo=one: L.block_boundary(I, H, z, o, None, n, C.byref(pp), Lo, None, None, None)
    assert call(I=None) == -1 and "null" in _err()
    assert call(Lo=None) == -1
    assert call(n=0) == -1
    assert call(n=33) == -3
    assert call(o=(C.c_int32 * 1)(0)) == -3 and "window" in _err()
    assert call(o=(C.c_int32 * 1)(257)) == -3
    for bad in (api.dlm_boundary_params(0.0, 8, 1, 0, 0), api.dlm_boundary_params(1.2, 0, 1, 0, 0),
                api.dlm_boundary_params(1.2, 8, -1, 0, 0), api.dlm_boundary_params(1.2, 8, 1, 4, 0),
                api.dlm_boundary_params(1.2, 8, 1, 0, 2)):
        assert call(pp=bad) == -1


def test_select_parallel_argument_errors():
    L = api.lib()
    one = C.c_void_p(16)
    p = api.dlm_select_params(0.8, 0.95, -16.0, 0)
    z = (C.c_int32 * 1)(0)
    bl = (C.c_int32 * 1)(8)

    def call(logits=one, vocab=100, dtype=1, n=1, pp=p, blen=bl, sel=one):
        return L.select_parallel(logits, vocab, dtype, one, one, one, one, z, z, blen, n, 99, C.byref(pp), 1, sel, one, None, None)

    assert call(logits=None) == -1 and call(sel=None) == -1
    assert call(n=0) == -1 and call(n=40) == -3
    assert call(dtype=2) == -1 and call(vocab=1) == -1
    assert call(pp=api.dlm_select_params(0.9, 0.8, -16.0, 0)) == -1 and "tau_high" in _err()
    assert call(pp=api.dlm_select_params(0.8, 0.95, -16.0, 3)) == -1
    assert call(blen=(C.c_int32 * 1)(257)) == -3 and call(blen=(C.c_int32 * 1)(-1)) == -3


def test_model_and_component_argument_errors():
    L = api.lib()
    one = C.c_void_p(16)
    h = C.c_void_p()
    cfg = api.dlm_config(2, 128, 4, 4, 32, 384, 1024, 1023, 0, 1e-5, 10000.0)
    assert L.dlm_model_create(C.byref(cfg), None, None, C.byref(h)) == -1
    w = api.dlm_weights()
    assert L.dlm_model_create(C.byref(cfg), C.byref(w), None, C.byref(h)) == -1 and "null weight" in _err()
    for field, val, code in (("dtype", 5, -1), ("head_dim", 48, -2), ("n_kv_heads", 3, -2), ("mask_id", 1024, -1), ("vocab", 1, -2)):
        bad = api.dlm_config(2, 128, 4, 4, 32, 384, 1024, 1023, 0, 1e-5, 10000.0)
        setattr(bad, field, val)
        assert L.dlm_model_create(C.byref(bad), C.byref(w), None, C.byref(h)) == code, field
    bf = api.dlm_config(2, 128, 4, 4, 32, 392, 1024, 1023, 1, 1e-5, 10000.0)  # d_ffn not a multiple of 32
    assert L.dlm_model_create(C.byref(bf), C.byref(w), None, C.byref(h)) == -2
    assert L.dlm_state_create(None, 1, 1, 1, 1, C.byref(h)) == -1
    assert L.dlm_step(None, None, None) == -1
    assert L.dlm_state_reset(None, 0) == -1 and L.dlm_state_kv_len(None, 0) == -1
    assert L.dlm_vocab_stats(None, None, None, 1, 8, 0, 7, one, one, one, one, one, one, one, 1 << 20, None) == -1
    assert L.dlm_vocab_stats(one, None, None, 0, 8, 0, 7, one, one, one, one, one, one, one, 1 << 20, None) == -3
    assert L.dlm_vocab_stats(one, None, None, 4, 8, 0, 7, one, one, one, one, one, one, one, 8, None) == -3 and "workspace" in _err()
    assert L.dlm_vocab_stats(one, None, None, 4, 8, 0, 8, one, one, one, one, one, one, one, 1 << 20, None) == -1
    # the entry point that allocates nothing: same checks, and a row limit set by its file-scope scratch
    assert L.dlm_vocab_stats_static(None, None, None, 1, 8, 0, 7, one, one, one, one, one, one, None) == -1
    assert L.dlm_vocab_stats_static(one, None, None, 0, 8, 0, 7, one, one, one, one, one, one, None) == -3
    assert L.dlm_vocab_stats_static(one, None, None, 4097, 8, 0, 7, one, one, one, one, one, one, None) == -3 and "4096" in _err()
    assert L.dlm_vocab_stats_static(one, None, None, 4, 8, 0, 8, one, one, one, one, one, one, None) == -1
    assert L.dlm_gemm_nt(one, one, one, 4, 48, 64, 1, None) == -2
    assert L.dlm_gemm_nt(one, None, one, 4, 64, 64, 1, None) == -1
    assert L.dlm_attention(one, one, one, one, 4, 4, 4, 3, 32, 0, None) == -2
    assert L.dlm_attention(one, one, one, one, 4, 4, 4, 2, 48, 0, None) == -2
    assert L.dlm_vocab_stats_workspace(0) == 0 and L.dlm_vocab_stats_workspace(64) > 0


def test_committed_traffic_summary_feeds_the_bench_line():
    """bench.py takes roofline.traffic of the default workload from the committed counter summary: it must hold both figures, and
    they must be within a few per cent of the kernel's algorithmic bytes (more would mean re-reads from HBM)."""
    import sys
    if ROOT not in sys.path:
        sys.path.insert(0, ROOT)
    import bench
    t = bench.traffic_from_profile("llada8b_p256_g256")
    algorithmic = 2 * 24576 * 4096  # the gate/up weights of the 8B shape, bf16
    assert t is not None and 0.98 * algorithmic < t < 1.10 * algorithmic
