"""ctypes front end of the CPU oracle (oracle.cpp).

TEST INFRASTRUCTURE: imported only by tests, the smoke check and the benchmark's
cpu_baseline leg.  It does not import the GPU package, and the GPU package does
not import it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None

F32, BF16, F16 = 0, 1, 2
W8 = 3   # blob format only: see from_shape
ROUND_KV, ROUND_GEMM_IN, ROUND_ATTN_QP, ROUND_HEAD_IN, ROUND_F16 = 1, 2, 4, 8, 16


class OrcConfig(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in (
        "hidden", "n_layers", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab",
        "has_embed_and_head", "tied_lm_head", "blob_dtype", "max_batch", "max_seq")] + [
        ("rms_eps", ctypes.c_double), ("rope_theta", ctypes.c_double)]


def build(force: bool = False) -> str:
    src = os.path.join(_HERE, "oracle.cpp")
    if force or not os.path.exists(LIB_PATH) or os.path.getmtime(LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["g++", "-std=c++17", "-O2", "-fopenmp", "-shared", "-fPIC",
                               "-Wall", "-Wextra", "-o", LIB_PATH, src])
    return LIB_PATH


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(LIB_PATH)
        vp, u32, i32, dbl, u64 = (ctypes.c_void_p, ctypes.c_uint32, ctypes.c_int32,
                                  ctypes.c_double, ctypes.c_uint64)
        sig = {
            "orc_bf16_round": (dbl, [dbl]),
            "orc_bf16_bits": (ctypes.c_uint16, [ctypes.c_float]),
            "orc_f16_round": (dbl, [dbl]),
            "orc_f16_bits": (ctypes.c_uint16, [ctypes.c_float]),
            "orc_silu": (dbl, [dbl]),
            "orc_rmsnorm": (None, [vp, vp, u32, dbl, vp]),
            "orc_rope": (None, [vp, u32, u32, dbl, vp]),
            "orc_softmax": (None, [vp, u32, vp]),
            "orc_matvec": (None, [vp, ctypes.c_int, u32, u32, vp, vp]),
            "orc_attend": (None, [vp, vp, vp, u32, u32, ctypes.c_size_t, ctypes.c_int, vp]),
            "orc_argmax": (i32, [vp, u32]),
            "orc_blob_bytes": (u64, [ctypes.POINTER(OrcConfig)]),
            "orc_create": (vp, [ctypes.POINTER(OrcConfig), vp, u64]),
            "orc_destroy": (None, [vp]),
            "orc_kv_reset": (None, [vp, i32]),
            "orc_slot_len": (u32, [vp, u32]),
            "orc_kv_rows": (vp, [vp, u32, u32, ctypes.c_int]),
            "orc_step_token": (ctypes.c_int, [vp, u32, i32, u32, vp, vp]),
            "orc_prefill": (ctypes.c_int, [vp, u32, vp, u32, u32, vp, vp]),
            "orc_step_hidden": (ctypes.c_int, [vp, u32, vp, u32, vp]),
            "orc_set_threads": (None, [ctypes.c_int]),
            "orc_get_threads": (ctypes.c_int, []),
        }
        for name, (res, args) in sig.items():
            f = getattr(L, name)
            f.restype, f.argtypes = res, args
        _lib = L
    return _lib


def _d(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data


# ---- building blocks ---------------------------------------------------------

def bf16_round(v: float) -> float:
    return lib().orc_bf16_round(float(v))


def bf16_bits(f: float) -> int:
    return int(lib().orc_bf16_bits(float(np.float32(f))))


def f16_round(v: float) -> float:
    return lib().orc_f16_round(float(v))


def f16_bits(f: float) -> int:
    return int(lib().orc_f16_bits(float(np.float32(f))))


def silu(z: float) -> float:
    return lib().orc_silu(float(z))


def rmsnorm(x, g, eps: float):
    x, xp = _d(x)
    out = np.empty_like(x)
    if g is None:
        lib().orc_rmsnorm(xp, None, x.size, eps, out.ctypes.data)
    else:
        g, gp = _d(g)
        lib().orc_rmsnorm(xp, gp, x.size, eps, out.ctypes.data)
    return out


def rope(u, pos: int, theta: float):
    u, up = _d(u)
    out = np.empty_like(u)
    lib().orc_rope(up, u.size, pos, theta, out.ctypes.data)
    return out


def softmax(s):
    s, sp = _d(s)
    out = np.empty_like(s)
    lib().orc_softmax(sp, s.size, out.ctypes.data)
    return out


def matvec(w: np.ndarray, x, dtype: int = F32):
    """w: [rows, cols] float32 (dtype F32) or uint16 bit patterns (dtype BF16 / F16)."""
    w = np.ascontiguousarray(w)
    assert w.dtype == (np.float32 if dtype == F32 else np.uint16)
    x, xp = _d(x)
    y = np.empty(w.shape[0], dtype=np.float64)
    lib().orc_matvec(w.ctypes.data, dtype, w.shape[0], w.shape[1], xp, y.ctypes.data)
    return y


def attend(q, keys, vals, round_p: int = 0):
    """q [d]; keys, vals [n, d] -> softmax(q K^T / sqrt(d)) V.  round_p: 0 / 1 (bf16) / 2 (binary16)."""
    q, qp = _d(q)
    keys, kp = _d(keys)
    vals, vp = _d(vals)
    out = np.empty_like(q)
    lib().orc_attend(qp, kp, vp, keys.shape[0], q.size, keys.shape[1], int(round_p), out.ctypes.data)
    return out


def argmax(v) -> int:
    v, p = _d(v)
    return int(lib().orc_argmax(p, v.size))


def set_threads(n: int) -> None:
    lib().orc_set_threads(int(n))


def get_threads() -> int:
    return int(lib().orc_get_threads())


# ---- model -------------------------------------------------------------------

class OracleModel:
    """The fp64 reference model over a canonical weight blob (borrowed, kept alive here)."""

    def __init__(self, *, hidden, n_layers, n_q_heads, n_kv_heads, head_dim, ffn, vocab,
                 has_embed_and_head, tied_lm_head, blob_dtype, max_batch, max_seq,
                 rms_eps, rope_theta, blob: np.ndarray):
        self.cfg = OrcConfig(hidden, n_layers, n_q_heads, n_kv_heads, head_dim, ffn, vocab,
                             int(has_embed_and_head), int(tied_lm_head), blob_dtype,
                             max_batch, max_seq, rms_eps, rope_theta)
        self.blob = np.ascontiguousarray(blob)
        self.h = lib().orc_create(ctypes.byref(self.cfg), self.blob.ctypes.data, self.blob.nbytes)
        if not self.h:
            raise ValueError("oracle: config/blob mismatch (expected %d bytes, got %d)" % (
                lib().orc_blob_bytes(ctypes.byref(self.cfg)), self.blob.nbytes))

    def close(self):
        if self.h:
            lib().orc_destroy(self.h)
            self.h = None

    def __del__(self):
        self.close()

    def kv_reset(self, slot: int = -1):
        lib().orc_kv_reset(self.h, slot)

    def slot_len(self, slot: int) -> int:
        return lib().orc_slot_len(self.h, slot)

    def step_token(self, slot: int, token: int, flags: int = 0, want_logits: bool = True):
        V = self.cfg.vocab
        logits = np.empty(V, dtype=np.float64) if want_logits else None
        nxt = ctypes.c_int32(-2)
        rc = lib().orc_step_token(self.h, slot, int(token), flags,
                                  logits.ctypes.data if want_logits else None,
                                  ctypes.byref(nxt) if want_logits else None)
        if rc:
            raise RuntimeError(f"oracle step_token rc={rc}")
        return logits, (nxt.value if want_logits else None)

    def prefill(self, slot: int, tokens, flags: int = 0):
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        logits = np.empty(self.cfg.vocab, dtype=np.float64)
        nxt = ctypes.c_int32(-2)
        rc = lib().orc_prefill(self.h, slot, t.ctypes.data, t.size, flags, logits.ctypes.data,
                               ctypes.byref(nxt))
        if rc:
            raise RuntimeError(f"oracle prefill rc={rc}")
        return logits, nxt.value

    def step_hidden(self, slot: int, x, flags: int = 0):
        x, xp = _d(x)
        y = np.empty(self.cfg.hidden, dtype=np.float64)
        rc = lib().orc_step_hidden(self.h, slot, xp, flags, y.ctypes.data)
        if rc:
            raise RuntimeError(f"oracle step_hidden rc={rc}")
        return y

    def kv_rows(self, layer: int, slot: int, which: int, n: int | None = None):
        """[n, Dkv] copy of the cached K (which=0) or V (which=1) rows."""
        n = self.slot_len(slot) if n is None else n
        dkv = self.cfg.n_kv_heads * self.cfg.head_dim
        p = lib().orc_kv_rows(self.h, layer, slot, which)
        buf = (ctypes.c_double * (n * dkv)).from_address(p)
        return np.frombuffer(buf, dtype=np.float64).reshape(n, dkv).copy()


def _widen_w8_blob(shape, blob: np.ndarray) -> np.ndarray:
    """Weight-only 8-bit blob -> the fp32 blob of the same model.

    The format (canonical order as for the other dtypes): a matrix of a layer is rows x cols signed
    bytes q followed by rows fp32 scales s; embedding / LM head are bf16; gains fp32.  The model's
    weight is w[r, c] = s[r] * q[r, c] -- this line is the oracle's statement of what the 8-bit
    format means.  The scales carry 8 significant bits and |q| <= 127, so the product is exact in
    fp32 and the fp64 forward pass below sees exactly the weights the format defines.
    """
    H, d = shape.hidden, shape.head_dim
    Dq, Dkv, F, V = shape.n_q_heads * d, shape.n_kv_heads * d, shape.ffn, shape.vocab
    src = np.ascontiguousarray(blob).view(np.uint8)
    parts, off = [], 0

    def take(n, dt):
        nonlocal off
        a = np.frombuffer(src, dtype=dt, count=n, offset=off)
        off += n * np.dtype(dt).itemsize
        return a

    def bf16(n):
        return (take(n, np.uint16).astype(np.uint32) << 16).view(np.float32)

    def w8(rows, cols):
        q = take(rows * cols, np.int8).reshape(rows, cols)
        s = take(rows, np.float32)
        w = q.astype(np.float64) * s.astype(np.float64)[:, None]
        w32 = w.astype(np.float32)
        assert np.array_equal(w32.astype(np.float64), w), "scale * byte is not exact in fp32"
        return w32.reshape(-1)

    if shape.has_embed_and_head:
        parts.append(bf16(V * H))
    for _ in range(shape.n_layers):
        parts += [take(H, np.float32), w8(Dq, H), w8(Dkv, H), w8(Dkv, H), take(d, np.float32), take(d, np.float32),
                  w8(H, Dq), take(H, np.float32), w8(F, H), w8(F, H), w8(H, F)]
    if shape.has_embed_and_head:
        parts.append(take(H, np.float32))
        if not shape.tied_lm_head:
            parts.append(bf16(V * H))
    assert off == src.size, "8-bit blob size does not match the shape"
    return np.concatenate(parts).view(np.uint8)


def from_shape(shape, blob: np.ndarray, max_batch: int, max_seq: int) -> OracleModel:
    """Build from an object with the shape field names used throughout (hidden, n_layers, ...).
    A weight-only 8-bit blob (dtype W8) is widened to fp32 first (exactly: _widen_w8_blob)."""
    if shape.dtype == W8:
        blob = _widen_w8_blob(shape, blob)
        return OracleModel(hidden=shape.hidden, n_layers=shape.n_layers, n_q_heads=shape.n_q_heads,
                           n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim, ffn=shape.ffn,
                           vocab=shape.vocab, has_embed_and_head=shape.has_embed_and_head,
                           tied_lm_head=shape.tied_lm_head, blob_dtype=F32,
                           max_batch=max_batch, max_seq=max_seq, rms_eps=shape.rms_eps,
                           rope_theta=shape.rope_theta, blob=blob)
    return OracleModel(hidden=shape.hidden, n_layers=shape.n_layers, n_q_heads=shape.n_q_heads,
                       n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim, ffn=shape.ffn,
                       vocab=shape.vocab, has_embed_and_head=shape.has_embed_and_head,
                       tied_lm_head=shape.tied_lm_head, blob_dtype=shape.dtype,
                       max_batch=max_batch, max_seq=max_seq, rms_eps=shape.rms_eps,
                       rope_theta=shape.rope_theta, blob=blob)
