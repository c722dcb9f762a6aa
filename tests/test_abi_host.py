"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
declared symbol, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import numpy as np
import pytest

import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def nnc():
    from paper_2512_21571_amd import binding
    binding.lib()
    return binding


def test_library_exports_every_declared_symbol(nnc):
    header = open(os.path.join(ROOT, "include", "nnc.h")).read()
    declared = set(re.findall(r"\b(nnc_[a-z_]+)\s*\(", header))
    assert declared == set(nnc.EXPORTS)
    for name in declared:
        assert getattr(nnc.lib(), name) is not None


def test_binding_constants_match_the_header(nnc):
    """The Python binding restates the option and status codes of the header: same values."""
    header = open(os.path.join(ROOT, "include", "nnc.h")).read()
    opts = dict(re.findall(r"\bNNC_(OPT_[A-Z_]+)\s*=\s*(\d+)", header))
    assert len(opts) >= 7
    for name, value in opts.items():
        assert getattr(nnc, name) == int(value), name
    codes = dict(re.findall(r"\bNNC_(OK|E_[A-Z_]+)\s*=\s*(\d+)", header))
    assert len(codes) == 8
    for name, value in codes.items():
        assert getattr(nnc, name) == int(value), name


def test_blob_bytes_matches_generator_for_all_benchmark_shapes(nnc):
    for shape in synth.SHAPES.values():
        cfg = nnc.make_config(shape, 1, 64)
        assert nnc.blob_bytes(cfg) == synth.blob_offsets(shape)[1], shape.name


def _create(nnc, cfg, blob):
    h = ctypes.c_void_p()
    st = nnc.lib().nnc_model_create(ctypes.byref(cfg) if cfg is not None else None,
                                    blob.ctypes.data if blob is not None else None,
                                    blob.nbytes if blob is not None else 0, None, ctypes.byref(h))
    assert not h.value or st == nnc.OK
    return st


def test_create_rejects_bad_arguments_before_any_device_work(nnc):
    shape = synth.SHAPES["qwen3-0.6b"]
    blob = np.zeros(64, np.uint8)
    assert _create(nnc, None, blob) == nnc.E_ARG
    cfg = nnc.make_config(shape, 1, 64)
    assert _create(nnc, cfg, None) == nnc.E_ARG
    assert _create(nnc, cfg, blob) == nnc.E_BLOB
    assert "bytes" in nnc.last_error()
    bad = nnc.make_config(shape, 1, 64)
    bad.struct_bytes = 12
    assert _create(nnc, bad, blob) == nnc.E_CONFIG
    for field, value in [("head_dim", 64), ("n_kv_heads", 3), ("hidden", 1000), ("vocab", 1001),
                         ("max_batch", 0), ("compute_dtype", 7)]:
        bad = nnc.make_config(shape, 1, 64)
        setattr(bad, field, value)
        assert _create(nnc, bad, blob) == nnc.E_CONFIG, field
        assert nnc.blob_bytes(bad) == 0
    f32_from_bf16 = nnc.make_config(shape, 1, 64, compute_dtype=nnc.F32)
    assert _create(nnc, f32_from_bf16, blob) == nnc.E_CONFIG
    # weight-only 8-bit blobs compute in bf16 only and need hidden / ffn in multiples of 64
    w8 = synth.ModelShape("w8", hidden=128, n_layers=1, n_q_heads=2, n_kv_heads=1, head_dim=128, ffn=192,
                          vocab=64, dtype=synth.W8)
    assert nnc.blob_bytes(nnc.make_config(w8, 1, 64)) == synth.blob_offsets(w8)[1]
    assert nnc.blob_bytes(nnc.make_config(w8, 1, 64, compute_dtype=nnc.F16)) == 0
    assert nnc.blob_bytes(nnc.make_config(w8.scaled(hidden=96), 1, 64)) == 0
    assert nnc.blob_bytes(nnc.make_config(w8.scaled(ffn=160), 1, 64)) == 0


def test_null_model_arguments(nnc):
    L = nnc.lib()
    assert L.nnc_kv_reset(None, 0) == nnc.E_ARG
    assert L.nnc_prefill(None, 0, None, 1, None, None) == nnc.E_ARG
    assert L.nnc_decode_step(None, None, None, 1, None, None) == nnc.E_ARG
    assert L.nnc_profile_begin(None) == nnc.E_ARG
    L.nnc_model_destroy(None)
