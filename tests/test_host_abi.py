"""Host-side checks of the C ABI that need no GPU: every declared symbol is exported,
the packed-block format agrees with the oracle's own offset function, sizing queries and
argument errors behave as include/ls_stage.h says."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import synth
from oracle import stage_oracle as so
from paper_2502_09922_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ls_stage.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ls_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    names = declared_functions()
    assert len(names) >= 18
    for n in names:
        assert hasattr(b.lib, n), n
    assert sorted(b.EXPORTED) == names


@pytest.mark.parametrize("name", ["tiny_f32", "llama7b", "llama13b", "llama70b"])
def test_block_format_matches_the_oracles_layout(name):
    s = synth.CONFIGS[name]
    cfg = b.make_cfg(s, 4, 64, 64)
    off, nb = C.c_size_t(), C.c_size_t()
    for layer, lay, order in [
        (0, so.layer_block_layout(s), synth.TENSOR_ORDER_LAYER),
        (s.n_layers_total - 1, so.layer_block_layout(s), synth.TENSOR_ORDER_LAYER),
        (-1, so.embed_block_layout(s), ("embed",)),
        (s.n_layers_total, so.head_block_layout(s), synth.TENSOR_ORDER_HEAD),
    ]:
        assert b.ls_block_tensor_count(C.byref(cfg), layer) == len(order)
        assert b.ls_block_bytes(C.byref(cfg), layer) == lay["__bytes__"][0]
        for i, tname in enumerate(order):
            assert b.ls_block_tensor(C.byref(cfg), layer, i, C.byref(off), C.byref(nb)) == 0
            assert off.value == lay[tname][0]
            assert nb.value == int(np.prod(lay[tname][1])) * s.itemsize


def test_pack_block_roundtrips_through_the_oracle_reader():
    s = synth.StageShape("bf16", 2, 40, 4, 2, 6, 22, 50)  # sizes that need padding
    cfg = b.make_cfg(s, 2, 16, 16)
    t = synth.layer_tensors(s, 7, 1)
    buf = b.pack_block(cfg, 1, [t[n] for n in synth.TENSOR_ORDER_LAYER])
    got = so.unpack_block(s, so.layer_block_layout(s), buf)
    for n in t:
        np.testing.assert_array_equal(got[n], so.decode_values(t[n]))
    with pytest.raises(ValueError):
        b.pack_block(cfg, 1, [t["wo"]])


def test_sizing_queries():
    s = synth.CONFIGS["llama7b"]
    cfg = b.make_cfg(s, 8, 640, 4096)
    assert b.ls_stage_slab_bytes(C.byref(cfg), 8, 16) == 8 * 202383360 * 2
    assert b.ls_stage_kv_bytes(C.byref(cfg), 8, 16) == 8 * 8 * 32 * 640 * 128 * 2
    whole = b.ls_stage_slab_bytes(C.byref(cfg), 0, 32)
    assert whole == 32 * 202383360 * 2 + 2 * 32000 * 4096 * 2 + 4096 * 2
    assert b.ls_stage_workspace_bytes(C.byref(cfg), 8, 16) > 4096 * 4096 * 4
    # invalid spans and shapes size to zero
    assert b.ls_stage_slab_bytes(C.byref(cfg), 5, 5) == 0
    assert b.ls_stage_slab_bytes(C.byref(cfg), 0, 33) == 0
    bad = b.make_cfg(s.with_(n_kv_heads=5), 8, 640, 4096)
    assert b.ls_stage_workspace_bytes(C.byref(bad), 0, 1) == 0
    assert b.ls_block_bytes(C.byref(cfg), 33) == 0 and b.ls_block_bytes(C.byref(cfg), -2) == 0
    novocab = b.make_cfg(s.with_(vocab=0), 8, 640, 4096)
    assert b.ls_block_bytes(C.byref(novocab), -1) == 0


def test_argument_errors_are_reported_before_any_device_work():
    s = synth.CONFIGS["tiny_f32"]
    cfg = b.make_cfg(s, 1, 40, 32)
    h = C.c_void_p()
    assert b.ls_stage_create(C.byref(cfg), 0, 2, None, 0, None, 0, C.byref(h)) == b.LS_ERR_INVALID_ARG
    assert b"NULL" in b.ls_last_error()
    assert b.ls_stage_create(C.byref(cfg), 1, 1, 256, 1 << 30, 256, 1 << 30, C.byref(h)) == b.LS_ERR_BLOCK_RANGE
    assert b.ls_stage_create(C.byref(cfg), 0, 2, 256, 16, 512, 1 << 30, C.byref(h)) == b.LS_ERR_OOM
    assert b.ls_stage_create(C.byref(cfg), 0, 2, 257, 1 << 30, 512, 1 << 30, C.byref(h)) == b.LS_ERR_INVALID_ARG
    wrong = b.make_cfg(s, 1, 40, 32)
    wrong.abi_version = 99
    assert b.ls_stage_create(C.byref(wrong), 0, 2, 256, 1 << 30, 512, 1 << 30, C.byref(h)) == b.LS_ERR_INVALID_ARG
    assert h.value is None
    assert b.ls_stage_prefill(None, None, None, None, 1, 1, None, None, None, None) == b.LS_ERR_INVALID_ARG
    assert b.ls_stage_decode(None, None, 1, 0, None, None, None, None) == b.LS_ERR_INVALID_ARG
    assert b.ls_stage_load_block(None, None, 0, None) == b.LS_ERR_INVALID_ARG
    assert b.ls_stage_block_bytes(None, 0) == 0
    off, nb = C.c_size_t(), C.c_size_t()
    assert b.ls_block_tensor(C.byref(cfg), 0, 6, C.byref(off), C.byref(nb)) == b.LS_ERR_INVALID_ARG


def test_pipeline_argument_errors_need_no_gpu():
    h = C.c_void_p()
    assert b.ls_pipeline_create(None, 1, C.byref(h)) == b.LS_ERR_INVALID_ARG
    none = (C.c_void_p * 1)(None)
    assert b.ls_pipeline_create(none, 1, C.byref(h)) == b.LS_ERR_INVALID_ARG
    assert b.ls_pipeline_create(none, 0, C.byref(h)) == b.LS_ERR_INVALID_ARG
    assert h.value is None
    assert b.ls_pipeline_run(None, 0, None, 1, None) == b.LS_ERR_INVALID_ARG
    assert b.ls_stage_info(None, None, None, None) == b.LS_ERR_INVALID_ARG
    b.ls_pipeline_destroy(None)  # a no-op


def test_measurement_probes_reject_bad_arguments_without_a_gpu():
    assert b.ls_probe_read_gbps(None, 1 << 20, 1, None, None) < 0
    assert b.ls_probe_read_gbps(C.c_void_p(4096), 8, 1, None, None) < 0      # fewer than 16 bytes
    assert b.ls_probe_read_gbps(C.c_void_p(4100), 1 << 20, 1, None, None) < 0  # not 16-byte aligned
    assert b.ls_probe_read_gbps(C.c_void_p(4096), 1 << 20, 0, None, None) < 0
    assert b.ls_probe_mfma_tflops(0, 1, None, None) < 0
    assert b.ls_probe_mfma_tflops(10, 0, None, None) < 0
    assert b"ls_probe" in b.lib.ls_last_error()
