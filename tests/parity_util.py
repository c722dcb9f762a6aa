"""Shared helpers for GPU-vs-oracle parity tests (no arithmetic of the method here)."""
from __future__ import annotations

import numpy as np

import oracle
import synth

# Small Qwen3-shaped models the oracle finishes in well under a second per token.
# head_dim is 128 as in every benchmark configuration (the kernels are written for it).
SMALL_BF16 = synth.ModelShape("small-bf16", hidden=256, n_layers=2, n_q_heads=4, n_kv_heads=2,
                              head_dim=128, ffn=512, vocab=1024, dtype=synth.BF16)
SMALL_G4 = synth.ModelShape("small-g4", hidden=320, n_layers=2, n_q_heads=8, n_kv_heads=2,
                            head_dim=128, ffn=608, vocab=2064, dtype=synth.BF16, tied_lm_head=False)
SMALL_F16 = synth.ModelShape("small-f16", hidden=256, n_layers=2, n_q_heads=4, n_kv_heads=2,
                             head_dim=128, ffn=512, vocab=1024, dtype=synth.F16)
SMALL_G4_F16 = synth.ModelShape("small-g4-f16", hidden=320, n_layers=2, n_q_heads=8, n_kv_heads=2,
                                head_dim=128, ffn=608, vocab=2064, dtype=synth.F16, tied_lm_head=False)
SMALL_F32 = synth.ModelShape("small-f32", hidden=256, n_layers=2, n_q_heads=4, n_kv_heads=2,
                             head_dim=128, ffn=512, vocab=1024, dtype=synth.F32)
SMALL_LAYER_F32 = synth.ModelShape("small-layer-f32", hidden=256, n_layers=1, n_q_heads=4, n_kv_heads=2,
                                   head_dim=128, ffn=512, vocab=0, has_embed_and_head=False,
                                   tied_lm_head=False, dtype=synth.F32)


def oracle_flags(shape, mirrored_prefill: bool = False) -> int:
    f = 0
    if shape.dtype != synth.F32:
        f |= oracle.ROUND_KV
        if mirrored_prefill:
            f |= oracle.ROUND_GEMM_IN | oracle.ROUND_ATTN_QP
        if shape.dtype == synth.F16:
            f |= oracle.ROUND_F16          # every rounding point in binary16 instead of bf16
    return f


def rel_inf(got: np.ndarray, want: np.ndarray) -> float:
    """max |g - o| / max |o| (infinity-norm relative error of one row)."""
    return float(np.abs(got - want).max() / np.abs(want).max())


def top2_margin(logits: np.ndarray) -> float:
    part = np.partition(logits, -2)
    return float(part[-1] - part[-2])


# The library's documented blocking of a prompt call on the large-block path (include/nnc.h,
# NNC_OPT_PREFILL_EXACT = 0), restated here for the tests: blocks of up to 4096 tokens (or what
# NNC_OPT_PREFILL_BLOCK asks for); a call
# of more than 512 tokens runs its last 16 tokens through the three-piece (fp32-grade) path; a
# block of more than 512 tokens carries one bf16 piece per matrix-core input, else two.
PREFILL_BLOCK, PREFILL_TAIL, ONE_PIECE_ABOVE = 4096, 16, 512


def prefill_blocks(n: int, block: int = PREFILL_BLOCK):
    """[(first token, tokens, pieces)] of a default-mode prompt call of n tokens."""
    head = n - PREFILL_TAIL if n > ONE_PIECE_ABOVE else n
    out, t0 = [], 0
    while t0 < head:
        nb = min(block, head - t0)
        out.append((t0, nb, 1 if nb > ONE_PIECE_ABOVE else 2))
        t0 += nb
    if head < n:
        out.append((head, n - head, 3))
    return out


def oracle_prefill_like_library(o, slot, toks, shape, block: int = PREFILL_BLOCK):
    """The oracle's prompt pass with the library's rounding points mirrored block by block."""
    res = None
    for t0, nb, pieces in prefill_blocks(len(toks), block):
        res = o.prefill(slot, toks[t0:t0 + nb], oracle_flags(shape, mirrored_prefill=pieces == 1))
    return res
