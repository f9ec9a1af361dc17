"""Host-side checks that need no GPU: the shared library loads, exports every symbol the public header
declares, and its host-only entry points validate their arguments."""
import ctypes as C
import os
import re

import pytest

import synth
from paper_2604_27476_amd import binding, buildlib as build_mod

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(build_mod.lib_path()):
        build_mod.build(force=True)
    return binding.load_library()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "edgefm.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(edgefm_[a-z0-9_]+)\s*\(", header))
    assert declared, "no declarations parsed"
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in edgefm.h but not exported"
    assert declared == set(binding.EXPORTS)


def test_config_struct_matches_header_layout():
    # 8 x u32, 2 x float, 4 x u32
    assert C.sizeof(binding.edgefm_config) == 14 * 4
    assert C.sizeof(binding.edgefm_weights) == 10 * C.sizeof(C.c_void_p)


def test_query_sizes_accounts_for_weights_and_kv(lib):
    for shape in (synth.TINY, synth.QWEN_0P5B, synth.QWEN_7B):
        cfg = binding.make_config(shape)
        n = binding.edgefm_query_sizes(cfg)
        kv = shape.max_seq_len * shape.kv_bytes_per_context_token()
        assert n >= shape.weight_bytes_per_token() + kv
        assert n < 4 * (shape.weight_bytes_per_token() + kv) + (2 << 30)


@pytest.mark.parametrize("field,value", [
    ("n_layers", 0), ("hidden", 0), ("hidden", 260), ("head_dim", 96), ("n_kv_heads", 3), ("n_q_heads", 18),
    ("weight_dtype", 0), ("kv_dtype", 7), ("max_seq_len", 0), ("vocab", 0), ("intermediate", 100),
    ("hidden", 1 << 20),
])
def test_query_sizes_rejects_unsupported_configs(lib, field, value):
    cfg = binding.make_config(synth.TINY)
    setattr(cfg, field, value)
    n = C.c_size_t(0)
    assert lib.edgefm_query_sizes(C.byref(cfg), C.byref(n)) == binding.EDGEFM_ERR_INVALID_ARG


def test_null_arguments_are_errors_not_crashes(lib):
    n = C.c_size_t(0)
    cfg = binding.make_config(synth.TINY)
    assert lib.edgefm_query_sizes(None, C.byref(n)) == binding.EDGEFM_ERR_INVALID_ARG
    assert lib.edgefm_query_sizes(C.byref(cfg), None) == binding.EDGEFM_ERR_INVALID_ARG
    assert lib.edgefm_prefill(None, None, 0, None, 0, None, None) == binding.EDGEFM_ERR_INVALID_ARG
    assert lib.edgefm_decode_step(None, 0, None, None) == binding.EDGEFM_ERR_INVALID_ARG
    assert lib.edgefm_kv_reset(None, 0) == binding.EDGEFM_ERR_INVALID_ARG
    assert lib.edgefm_kv_len(None) == 0
    lib.edgefm_model_free(None)
    h = C.c_void_p()
    assert lib.edgefm_model_load(C.byref(cfg), None, None, 0, None, C.byref(h)) == binding.EDGEFM_ERR_INVALID_ARG
    assert not h.value


def test_vocab_subset_rejects_null_handle(lib):
    import ctypes as C
    ids = (C.c_int32 * 2)(1, 2)
    assert lib.edgefm_set_vocab_subset(None, ids, 2) == binding.EDGEFM_ERR_INVALID_ARG


def test_strerror_covers_every_status(lib):
    seen = set()
    for code in range(0, -7, -1):
        msg = lib.edgefm_strerror(code).decode()
        assert msg and msg != "unknown status"
        seen.add(msg)
    assert len(seen) == 7
    assert lib.edgefm_strerror(-99).decode() == "unknown status"


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "lib_path", lambda: str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError, match="not found"):
        binding.load_library()
