"""ctypes binding of include/nnc.h.  Argument marshalling only: every step of the
forward pass runs in the library's HIP kernels.  PyTorch supplies device memory
(through the allocator hooks) and the stream; there is no CPU or PyTorch fallback.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import _build

OK, E_ARG, E_CONFIG, E_BLOB, E_NOMEM, E_KV_FULL, E_DEVICE, E_STATE = range(8)
F32, BF16, F16 = 0, 1, 2
W8 = 3   # blob dtype only (weight-only 8 bits); computes in BF16
OPT_GRAPH, OPT_PREFILL_EXACT, OPT_PERSISTENT, OPT_STAGE_TRACE, OPT_PREFILL_TILE, OPT_SPIN_LIMIT = 0, 1, 2, 3, 4, 5
OPT_PREFILL_ATTN = 6
OPT_FUSE_QK = 7
OPT_TAIL_OVERLAP = 8
OPT_PREFILL_BLOCK = 9
OPT_PLANNER = 10
OPT_FUSE_NORM = 11
OPT_DECODE_PIECES = 12
OPT_PREFILL_KSLICES = 13

# every symbol include/nnc.h declares
EXPORTS = [
    "nnc_model_create", "nnc_model_destroy", "nnc_prefill", "nnc_decode_step", "nnc_decode_step_static",
    "nnc_decode_greedy",
    "nnc_kv_reset", "nnc_synchronize", "nnc_slot_len", "nnc_prefill_hidden", "nnc_decode_step_hidden", "nnc_kv_read",
    "nnc_set_option", "nnc_profile_begin", "nnc_profile_end", "nnc_stage_trace", "nnc_blob_bytes",
    "nnc_last_error", "nnc_plan_prefill_gemm_query", "nnc_plan_skinny_gemm_query",
]


class NncConfig(ctypes.Structure):
    _fields_ = [("struct_bytes", ctypes.c_uint32)] + [(n, ctypes.c_uint32) for n in (
        "hidden", "n_layers", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab")] + [
        ("rms_eps", ctypes.c_float), ("rope_theta", ctypes.c_float)] + [(n, ctypes.c_uint32) for n in (
            "has_embed_and_head", "tied_lm_head", "blob_dtype", "compute_dtype", "max_batch", "max_seq")]


ALLOC_FN = ctypes.CFUNCTYPE(ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p)
FREE_FN = ctypes.CFUNCTYPE(None, ctypes.c_void_p, ctypes.c_void_p)


class NncDevice(ctypes.Structure):
    _fields_ = [("alloc", ALLOC_FN), ("free", FREE_FN), ("ctx", ctypes.c_void_p), ("stream", ctypes.c_void_p)]


class NncKernelStat(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 48), ("launches", ctypes.c_uint64), ("total_ms", ctypes.c_double),
                ("bytes", ctypes.c_double), ("flops", ctypes.c_double)]


class NncGemmPlan(ctypes.Structure):
    _fields_ = [("tile_rows", ctypes.c_uint32), ("tile_cols", ctypes.c_uint32), ("tile_code", ctypes.c_int32),
                ("k_slices", ctypes.c_uint32), ("workgroups", ctypes.c_uint32), ("t_comp_us", ctypes.c_double),
                ("t_mem_us", ctypes.c_double), ("t_us", ctypes.c_double), ("candidates", ctypes.c_uint32),
                ("rejected_by_capacity", ctypes.c_uint32)]


class NncError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"nnc status {status}: {message}")
        self.status = status


_lib = None


def lib():
    """Load libnnc.so (building it first only if no built library exists)."""
    global _lib
    if _lib is None:
        # PyTorch ships its own HIP runtime (soname libamdhip64.so.7).  Import it first so
        # that libnnc.so binds to that already-loaded runtime: two HIP runtimes in one
        # process cannot both own the device.
        import torch  # noqa: F401
        if not os.path.exists(_build.LIB_PATH):
            _build.build(True)
        L = ctypes.CDLL(_build.LIB_PATH)   # raises OSError if the library cannot be loaded
        vp, u32, i32 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_int32
        P = ctypes.POINTER
        sig = {
            "nnc_model_create": (i32, [P(NncConfig), vp, ctypes.c_size_t, P(NncDevice), P(vp)]),
            "nnc_model_destroy": (None, [vp]),
            "nnc_prefill": (i32, [vp, u32, vp, u32, vp, vp]),
            "nnc_decode_step": (i32, [vp, vp, vp, u32, vp, vp]),
            "nnc_decode_step_static": (i32, [vp, vp, vp, u32, vp, vp]),
            "nnc_decode_greedy": (i32, [vp, vp, vp, u32, u32, vp, vp]),
            "nnc_kv_reset": (i32, [vp, i32]),
            "nnc_synchronize": (i32, [vp]),
            "nnc_slot_len": (i32, [vp, u32, P(u32)]),
            "nnc_prefill_hidden": (i32, [vp, u32, vp, u32, vp]),
            "nnc_decode_step_hidden": (i32, [vp, vp, vp, u32, vp]),
            "nnc_kv_read": (i32, [vp, u32, u32, u32, u32, u32, vp]),
            "nnc_set_option": (i32, [vp, i32, i32]),
            "nnc_profile_begin": (i32, [vp]),
            "nnc_profile_end": (i32, [vp, P(NncKernelStat), u32, P(u32)]),
            "nnc_stage_trace": (i32, [vp, vp, u32, P(u32), P(u32)]),
            "nnc_blob_bytes": (ctypes.c_uint64, [P(NncConfig)]),
            "nnc_last_error": (ctypes.c_char_p, []),
            "nnc_plan_prefill_gemm_query": (i32, [u32, u32, u32, u32, u32, u32, u32, P(NncGemmPlan)]),
            "nnc_plan_skinny_gemm_query": (i32, [u32, u32, u32, u32, u32, u32, u32, P(NncGemmPlan)]),
        }
        for name, (res, args) in sig.items():
            f = getattr(L, name)
            f.restype, f.argtypes = res, args
        _lib = L
    return _lib


def last_error() -> str:
    return lib().nnc_last_error().decode()


def _check(st: int):
    if st != OK:
        raise NncError(st, last_error())


def make_config(shape, max_batch: int, max_seq: int, compute_dtype: int | None = None) -> NncConfig:
    """shape: any object with the field names of nnc_config (hidden, n_layers, ...) and `dtype`."""
    return NncConfig(ctypes.sizeof(NncConfig), shape.hidden, shape.n_layers, shape.n_q_heads,
                     shape.n_kv_heads, shape.head_dim, shape.ffn, shape.vocab, shape.rms_eps,
                     shape.rope_theta, int(shape.has_embed_and_head), int(shape.tied_lm_head),
                     shape.dtype, (BF16 if shape.dtype == W8 else shape.dtype) if compute_dtype is None else compute_dtype,
                     max_batch, max_seq)


def blob_bytes(cfg: NncConfig) -> int:
    return int(lib().nnc_blob_bytes(ctypes.byref(cfg)))


def plan_prefill_gemm(rows, k, n_tokens, pieces, epilogue, max_k_slices=1, n_cus=256) -> NncGemmPlan:
    out = NncGemmPlan()
    _check(lib().nnc_plan_prefill_gemm_query(rows, k, n_tokens, pieces, epilogue, max_k_slices, n_cus, ctypes.byref(out)))
    return out


def plan_skinny_gemm(rows, k, n_seq, pieces, epilogue, max_k_slices=1, n_cus=256) -> NncGemmPlan:
    out = NncGemmPlan()
    _check(lib().nnc_plan_skinny_gemm_query(rows, k, n_seq, pieces, epilogue, max_k_slices, n_cus, ctypes.byref(out)))
    return out


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _u32(a):
    return np.ascontiguousarray(a, dtype=np.uint32)


class Model:
    """A model on cuda:0.  Device memory comes from torch's allocator, work runs on a
    torch stream of default priority; outputs are torch tensors on that stream."""

    def __init__(self, shape, blob: np.ndarray, max_batch: int, max_seq: int,
                 compute_dtype: int | None = None, device: str = "cuda:0"):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("nnc needs an MI355X: torch.cuda.is_available() is False")
        self.torch = torch
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.stream = torch.cuda.Stream(device=self.device)
        self.cfg = make_config(shape, max_batch, max_seq, compute_dtype)
        self._held = {}

        def _alloc(nbytes, _ctx):
            try:
                t = torch.empty(int(nbytes), dtype=torch.uint8, device=self.device)
            except Exception:
                return None
            self._held[t.data_ptr()] = t
            return t.data_ptr()

        def _free(p, _ctx):
            self._held.pop(p, None)

        self._alloc_cb, self._free_cb = ALLOC_FN(_alloc), FREE_FN(_free)
        self._dev = NncDevice(self._alloc_cb, self._free_cb, None, self.stream.cuda_stream)
        blob = np.ascontiguousarray(blob)
        h = ctypes.c_void_p()
        _check(lib().nnc_model_create(ctypes.byref(self.cfg), blob.ctypes.data, blob.nbytes,
                                      ctypes.byref(self._dev), ctypes.byref(h)))
        self.h = h
        self.V, self.H = self.cfg.vocab, self.cfg.hidden

    # -- lifetime -----------------------------------------------------------------
    def close(self):
        if getattr(self, "h", None):
            lib().nnc_model_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _empty(self, shape, dtype):
        with self.torch.cuda.stream(self.stream):
            return self.torch.empty(shape, dtype=dtype, device=self.device)

    def synchronize(self):
        """Wait for the model's stream; raises NncError if a resident decode launch gave up."""
        _check(lib().nnc_synchronize(self.h))

    def _before(self):
        # inputs may have been produced on the caller's current stream
        self.stream.wait_stream(self.torch.cuda.current_stream(self.device))

    def _after(self):
        # outputs are consumed on the caller's current stream
        self.torch.cuda.current_stream(self.device).wait_stream(self.stream)

    # -- forward pass ---------------------------------------------------------------
    def prefill(self, slot: int, tokens, want_logits: bool = True):
        t = _i32(tokens)
        logits = self._empty((self.V,), self.torch.float32) if want_logits else None
        nxt = self._empty((1,), self.torch.int32)
        self._before()
        try:
            _check(lib().nnc_prefill(self.h, slot, t.ctypes.data, t.size,
                                     logits.data_ptr() if want_logits else None, nxt.data_ptr()))
        finally:
            self._after()
        return logits, nxt

    def decode_step(self, slots, tokens, want_logits: bool = True):
        s, t = _u32(slots), _i32(tokens)
        b = s.size
        logits = self._empty((b, self.V), self.torch.float32) if want_logits else None
        nxt = self._empty((b,), self.torch.int32)
        self._before()
        try:
            _check(lib().nnc_decode_step(self.h, s.ctypes.data, t.ctypes.data, b,
                                         logits.data_ptr() if want_logits else None, nxt.data_ptr()))
        finally:
            self._after()
        return logits, nxt

    def decode_step_static(self, slots, tokens, logits=None, nxt=None):
        """nnc_decode_step_static: the caller passes the output tensors (nothing is allocated,
        here or in the library); either may be None."""
        s, t = _u32(slots), _i32(tokens)
        self._before()
        try:
            _check(lib().nnc_decode_step_static(self.h, s.ctypes.data, t.ctypes.data, s.size,
                                                logits.data_ptr() if logits is not None else None,
                                                nxt.data_ptr() if nxt is not None else None))
        finally:
            self._after()
        return logits, nxt

    def decode_greedy(self, slots, first_tokens, n_steps: int, want_logits: bool = False):
        s, t = _u32(slots), _i32(first_tokens)
        b = s.size
        toks = self._empty((n_steps, b), self.torch.int32)
        logits = self._empty((n_steps, b, self.V), self.torch.float32) if want_logits else None
        self._before()
        try:
            _check(lib().nnc_decode_greedy(self.h, s.ctypes.data, t.ctypes.data, b, n_steps, toks.data_ptr(),
                                           logits.data_ptr() if want_logits else None))
        finally:
            self._after()
        return toks, logits

    def prefill_hidden(self, slot: int, x):
        """x: [n, hidden] float32 torch tensor on the device (or array-like, copied)."""
        x = self._as_dev(x)
        y = self._empty(tuple(x.shape), self.torch.float32)
        self._before()
        try:
            _check(lib().nnc_prefill_hidden(self.h, slot, x.data_ptr(), x.shape[0], y.data_ptr()))
        finally:
            self._after()
        return y

    def decode_step_hidden(self, slots, x):
        s = _u32(slots)
        x = self._as_dev(x)
        y = self._empty(tuple(x.shape), self.torch.float32)
        self._before()
        try:
            _check(lib().nnc_decode_step_hidden(self.h, s.ctypes.data, x.data_ptr(), s.size, y.data_ptr()))
        finally:
            self._after()
        return y

    def _as_dev(self, x):
        torch = self.torch
        if not isinstance(x, torch.Tensor):
            x = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
        with torch.cuda.stream(self.stream):
            x = x.to(self.device, dtype=torch.float32, non_blocking=False).contiguous()
        if x.dim() == 1:
            x = x[None]
        return x

    # -- state ------------------------------------------------------------------------
    def kv_reset(self, slot: int = -1):
        _check(lib().nnc_kv_reset(self.h, slot))

    def slot_len(self, slot: int) -> int:
        n = ctypes.c_uint32()
        _check(lib().nnc_slot_len(self.h, slot, ctypes.byref(n)))
        return n.value

    def kv_read(self, layer: int, slot: int, which: int, pos0: int, n: int):
        dkv = self.cfg.n_kv_heads * self.cfg.head_dim
        out = self._empty((n, dkv), self.torch.float32)
        self._before()
        try:
            _check(lib().nnc_kv_read(self.h, layer, slot, which, pos0, n, out.data_ptr()))
        finally:
            self._after()
        return out

    def set_option(self, opt: int, value: int):
        _check(lib().nnc_set_option(self.h, opt, value))

    def stage_trace(self):
        """[workgroups, points] uint64 wall-clock ticks (10 ns) of the traced decode step."""
        cap = 1024 * (8 * self.cfg.n_layers + 3)
        buf = np.zeros(cap, dtype=np.uint64)
        nwg, npts = ctypes.c_uint32(), ctypes.c_uint32()
        _check(lib().nnc_stage_trace(self.h, buf.ctypes.data, cap, ctypes.byref(nwg), ctypes.byref(npts)))
        return buf[: nwg.value * npts.value].reshape(nwg.value, npts.value)

    # -- per-kernel event timing ---------------------------------------------------------
    def profile_begin(self):
        _check(lib().nnc_profile_begin(self.h))

    def profile_end(self):
        cap = 32
        arr = (NncKernelStat * cap)()
        n = ctypes.c_uint32()
        _check(lib().nnc_profile_end(self.h, arr, cap, ctypes.byref(n)))
        return [dict(name=arr[i].name.decode(), launches=int(arr[i].launches), total_ms=arr[i].total_ms,
                     bytes=arr[i].bytes, flops=arr[i].flops) for i in range(n.value)]
