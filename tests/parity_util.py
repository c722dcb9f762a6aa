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
SMALL_F32 = synth.ModelShape("small-f32", hidden=256, n_layers=2, n_q_heads=4, n_kv_heads=2,
                             head_dim=128, ffn=512, vocab=1024, dtype=synth.F32)
SMALL_LAYER_F32 = synth.ModelShape("small-layer-f32", hidden=256, n_layers=1, n_q_heads=4, n_kv_heads=2,
                                   head_dim=128, ffn=512, vocab=0, has_embed_and_head=False,
                                   tied_lm_head=False, dtype=synth.F32)


def oracle_flags(shape, mirrored_prefill: bool = False) -> int:
    f = 0
    if shape.dtype == synth.BF16:
        f |= oracle.ROUND_KV
        if mirrored_prefill:
            f |= oracle.ROUND_GEMM_IN | oracle.ROUND_ATTN_QP
    return f


def rel_inf(got: np.ndarray, want: np.ndarray) -> float:
    """max |g - o| / max |o| (infinity-norm relative error of one row)."""
    return float(np.abs(got - want).max() / np.abs(want).max())


def top2_margin(logits: np.ndarray) -> float:
    part = np.partition(logits, -2)
    return float(part[-1] - part[-2])
