"""Seeded synthetic inputs for Qwen3-shaped decoder models.

This module holds no decoder arithmetic.  It defines the workload shapes, the
canonical weight-blob layout (a file format) and draws the random numbers that
fill it.  Tests feed the same blob to the CPU oracle and to the GPU library.

Stands in for the trained Qwen3-0.6B / 1.7B checkpoints and the short prompt of
the paper's evaluation (Section 4, experimental setup); the 4B / 8B shapes extend
the same family.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, replace

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsynth.so")
_lib = None

WEIGHT_SEED = 251221571
INPUT_SEED = 251221572

F32, BF16, F16 = 0, 1, 2
# weight-only 8-bit: the matrices of the layers as signed bytes with one fp32 scale per output row,
# embedding / LM head in bf16; activations and KV cache as for BF16
W8 = 3


def build(force: bool = False) -> str:
    """Compile synth.c with gcc (OpenMP) into libsynth.so next to it."""
    src = os.path.join(_HERE, "synth.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB_PATH, src, "-lm"])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB_PATH)
        u64, dbl, vp = ctypes.c_uint64, ctypes.c_double, ctypes.c_void_p
        lib.synth_normal_f32.argtypes = [u64, u64, u64, u64, dbl, vp]
        lib.synth_normal_bf16.argtypes = [u64, u64, u64, u64, dbl, vp]
        lib.synth_normal_f16.argtypes = [u64, u64, u64, u64, dbl, vp]
        lib.synth_uniform_i32.argtypes = [u64, u64, u64, u64, ctypes.c_uint32, vp]
        lib.synth_normal_w8.argtypes = [u64, u64, u64, u64, dbl, vp, vp]
        lib.synth_normal_w8.restype = None
        lib.synth_raw.argtypes = [u64, u64, u64]
        lib.synth_raw.restype = u64
        for f in (lib.synth_normal_f32, lib.synth_normal_bf16, lib.synth_normal_f16, lib.synth_uniform_i32):
            f.restype = None
        _lib = lib
    return _lib


@dataclass(frozen=True)
class ModelShape:
    """Hyper-parameters of one synthetic model (names follow the Qwen3 family)."""
    name: str
    hidden: int
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    has_embed_and_head: bool = True
    tied_lm_head: bool = True
    dtype: int = BF16            # blob dtype == compute dtype
    rms_eps: float = 1e-6
    rope_theta: float = 1e6

    @property
    def dq(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def dkv(self) -> int:
        return self.n_kv_heads * self.head_dim

    def scaled(self, **kw) -> "ModelShape":
        return replace(self, **kw)


V_QWEN3 = 151936
SHAPES = {
    # one decoder layer, fp32, hidden-state in / hidden-state out
    "layer-0.6b-f32": ModelShape("layer-0.6b-f32", 1024, 1, 16, 8, 128, 3072, 0,
                                 has_embed_and_head=False, tied_lm_head=False, dtype=F32),
    "qwen3-0.6b": ModelShape("qwen3-0.6b", 1024, 28, 16, 8, 128, 3072, V_QWEN3),
    # the paper's own 16-bit precision (IEEE binary16) at its smallest model
    "qwen3-0.6b-f16": ModelShape("qwen3-0.6b-f16", 1024, 28, 16, 8, 128, 3072, V_QWEN3, dtype=F16),
    "qwen3-1.7b": ModelShape("qwen3-1.7b", 2048, 28, 16, 8, 128, 6144, V_QWEN3),
    "qwen3-4b": ModelShape("qwen3-4b", 2560, 36, 32, 8, 128, 9728, V_QWEN3),
    "qwen3-8b": ModelShape("qwen3-8b", 4096, 36, 32, 8, 128, 12288, V_QWEN3, tied_lm_head=False),
    # weight-only 8-bit layers (not a format of the paper: a step beyond its 16-bit runs)
    "qwen3-8b-w8": ModelShape("qwen3-8b-w8", 4096, 36, 32, 8, 128, 12288, V_QWEN3, tied_lm_head=False, dtype=W8),
}


def blob_layout(s: ModelShape):
    """Canonical blob: list of (name, shape, is_gain) in storage order.

    Matrices are row-major [out, in] in the blob dtype; gains are always fp32.
    The ordinal of an entry is its tensor id for the generator.
    W8 blobs: a matrix of a layer is rows x cols signed bytes followed by rows fp32 scales (the
    weight is scale[row] * byte); embedding and LM head are bf16.
    """
    out = []
    if s.has_embed_and_head:
        out.append(("embed", (s.vocab, s.hidden), False))
    for l in range(s.n_layers):
        p = f"l{l}."
        out += [
            (p + "g_in", (s.hidden,), True),
            (p + "wq", (s.dq, s.hidden), False),
            (p + "wk", (s.dkv, s.hidden), False),
            (p + "wv", (s.dkv, s.hidden), False),
            (p + "g_q", (s.head_dim,), True),
            (p + "g_k", (s.head_dim,), True),
            (p + "wo", (s.hidden, s.dq), False),
            (p + "g_post", (s.hidden,), True),
            (p + "wgate", (s.ffn, s.hidden), False),
            (p + "wup", (s.ffn, s.hidden), False),
            (p + "wdown", (s.hidden, s.ffn), False),
        ]
    if s.has_embed_and_head:
        out.append(("g_final", (s.hidden,), True))
        if not s.tied_lm_head:
            out.append(("lm_head", (s.vocab, s.hidden), False))
    return out


def _layer_matrix(name: str) -> bool:
    return name[0] == "l" and name[1].isdigit()


def blob_offsets(s: ModelShape):
    """name -> (byte offset, shape, numpy dtype) and the total byte count."""
    esz = 4 if s.dtype == F32 else 2
    off, table = 0, {}
    for name, shape, is_gain in blob_layout(s):
        n = int(np.prod(shape))
        if is_gain:
            table[name] = (off, shape, np.float32)
            off += 4 * n
        elif s.dtype == W8 and _layer_matrix(name):
            table[name] = (off, shape, np.int8)
            table[name + ".scale"] = (off + n, (shape[0],), np.float32)
            off += n + 4 * shape[0]
        else:
            table[name] = (off, shape, np.float32 if s.dtype == F32 else np.uint16)
            off += esz * n
    return table, off


def make_blob(s: ModelShape, seed: int = WEIGHT_SEED, weight_std: float = 0.02,
              gain_jitter: float = 0.0) -> np.ndarray:
    """Fill the canonical blob: matrices ~ N(0, weight_std^2), gains 1.0.

    gain_jitter > 0 draws gains as 1 + jitter * N(0,1) instead (used by tests so
    that a dropped or misplaced gain is visible; the benchmark configs use 1.0).
    """
    lib = _load()
    table, total = blob_offsets(s)
    blob = np.empty(total, dtype=np.uint8)
    base = blob.ctypes.data
    for tid, (name, shape, is_gain) in enumerate(blob_layout(s)):
        off = table[name][0]
        n = int(np.prod(shape))
        if is_gain:
            g = np.frombuffer(blob, dtype=np.float32, count=n, offset=off)
            if gain_jitter > 0.0:
                lib.synth_normal_f32(seed, tid, 0, n, gain_jitter, base + off)
                g += 1.0
            else:
                g[:] = 1.0
        elif s.dtype == W8 and _layer_matrix(name):
            lib.synth_normal_w8(seed, tid, shape[0], shape[1], weight_std, base + off, base + off + n)
        elif s.dtype == F32:
            lib.synth_normal_f32(seed, tid, 0, n, weight_std, base + off)
        elif s.dtype == F16:
            lib.synth_normal_f16(seed, tid, 0, n, weight_std, base + off)
        else:
            lib.synth_normal_bf16(seed, tid, 0, n, weight_std, base + off)
    return blob


def blob_tensor(s: ModelShape, blob: np.ndarray, name: str) -> np.ndarray:
    """View of one tensor inside the blob (uint16 holds bf16 or binary16 bit patterns)."""
    table, _ = blob_offsets(s)
    off, shape, dt = table[name]
    return np.frombuffer(blob, dtype=dt, count=int(np.prod(shape)), offset=off).reshape(shape)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen stored bf16 bit patterns to fp32 (exact; a format conversion)."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


def f16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen stored binary16 bit patterns to fp32 (exact; a format conversion)."""
    return bits.view(np.float16).astype(np.float32)


def tokens(n: int, vocab: int, stream: int = 0, seed: int = INPUT_SEED) -> np.ndarray:
    """n token ids uniform in [0, vocab); one independent stream per sequence slot."""
    out = np.empty(n, dtype=np.int32)
    _load().synth_uniform_i32(seed, 1000 + stream, 0, n, vocab, out.ctypes.data)
    return out


def activations(rows: int, cols: int, stream: int = 0, seed: int = INPUT_SEED,
                std: float = 1.0) -> np.ndarray:
    """[rows, cols] fp32 ~ N(0, std^2) (hidden-state inputs of the one-layer config)."""
    out = np.empty((rows, cols), dtype=np.float32)
    _load().synth_normal_f32(seed, 2000 + stream, 0, rows * cols, std, out.ctypes.data)
    return out


def raw(seed: int, tensor: int, i: int) -> int:
    return int(_load().synth_raw(seed, tensor, i))
