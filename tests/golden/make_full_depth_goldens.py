"""Writes the full-depth expected values of the 4B / 8B workloads (CPU only, oracle only).

The fp64 oracle needs hours for these models, so it runs offline, here, and the GPU tests load
what it wrote.  This script imports nothing but the oracle, the seeded input generator and the
test helper that restates the library's documented prompt blocking; it never touches the GPU
library.

For one workload it runs slot 0 (token stream 0) of the full model at the full context:
the prompt pass, then `--steps` greedy decode steps, each fed the oracle's own previous token.
Stored per variant: fp32 copies of the fp64 logits of the prompt's last position and of every
decode step, the oracle's greedy tokens and top-2 margins.

Variants:
  plain     every position with the cache rounding only (ORC_ROUND_KV): the exact definition
            with a 16-bit cache
  mirrored  prompt blocks of more than 512 tokens additionally round the matrix-core inputs
            where the library's single-piece blocks do (parity_util.prefill_blocks)

Usage: python tests/golden/make_full_depth_goldens.py cfg3|cfg4 [--variants plain,mirrored]
       [--steps 8] [--threads N]          (cfg3: about 25 min per variant on 8 cores; cfg4: 1.5 h)
"""
from __future__ import annotations

import argparse
import hashlib
import os
import sys
import threading
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import oracle  # noqa: E402
import synth  # noqa: E402
from parity_util import oracle_flags, prefill_blocks, top2_margin  # noqa: E402

WORKLOADS = {"cfg3": ("qwen3-4b", 2048), "cfg4": ("qwen3-8b", 4096)}


def oracle_hash() -> str:
    with open(os.path.join(ROOT, "oracle", "oracle.cpp"), "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()


def golden_path(workload: str, variant: str) -> str:
    return os.path.join(HERE, f"{workload}_slot0_{variant}.npz")


def run_variant(o, slot, variant, shape, toks, steps, out, tag):
    fl = oracle_flags(shape)
    t0 = time.time()
    if variant == "plain":
        blocks = [(0, len(toks), 3)]
    else:
        blocks = prefill_blocks(len(toks))
    done = 0
    res = None
    for first, nb, pieces in blocks:
        bf = oracle_flags(shape, mirrored_prefill=(variant == "mirrored" and pieces == 1))
        # in pieces of 32 tokens so that progress is visible
        for c0 in range(first, first + nb, 32):
            n = min(32, first + nb - c0)
            res = o.prefill(slot, toks[c0:c0 + n], bf)
            done += n
            el = time.time() - t0
            print(f"[{tag}] prompt {done}/{len(toks)}  {el:7.0f} s  eta {el / done * (len(toks) + steps - done):7.0f} s",
                  flush=True)
    logits = np.empty((steps + 1, shape.vocab), np.float32)
    nxt = np.empty(steps + 1, np.int32)
    margin = np.empty(steps + 1, np.float64)
    lo, t = res
    logits[0], nxt[0], margin[0] = lo, t, top2_margin(lo)
    for s in range(steps):
        lo, t = o.step_token(slot, int(nxt[s]), fl)
        logits[s + 1], nxt[s + 1], margin[s + 1] = lo, t, top2_margin(lo)
        print(f"[{tag}] decode step {s + 1}/{steps}  token {t}  margin {margin[s + 1]:.3e}", flush=True)
    out[variant] = (logits, nxt, margin)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("workload", choices=sorted(WORKLOADS))
    ap.add_argument("--variants", default="plain,mirrored")
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--threads", type=int, default=0, help="OpenMP threads per variant (0: all cores / variants)")
    a = ap.parse_args()
    name, ctx = WORKLOADS[a.workload]
    variants = a.variants.split(",")
    shape = synth.SHAPES[name]
    # every variant runs in a thread of its own; each thread's OpenMP team takes its size
    # from the environment, which must be set before the library is loaded
    os.environ["OMP_NUM_THREADS"] = str(a.threads or max(1, (os.cpu_count() or 1) // len(variants)))
    print(f"{a.workload}: {name}, context {ctx}, {a.steps} decode steps, variants {variants}, "
          f"{oracle.get_threads()} threads each", flush=True)
    blob = synth.make_blob(shape)
    toks = synth.tokens(ctx, shape.vocab, stream=0)
    o = oracle.from_shape(shape, blob, len(variants), ctx + a.steps)
    out, th = {}, []
    for slot, v in enumerate(variants):
        th.append(threading.Thread(target=run_variant, args=(o, slot, v, shape, toks, a.steps, out, v)))
        th[-1].start()
    for t in th:
        t.join()
    for v in variants:
        logits, nxt, margin = out[v]
        np.savez(golden_path(a.workload, v), logits=logits, next=nxt, margin=margin,
                 shape=name, context=ctx, stream=0, weight_seed=synth.WEIGHT_SEED,
                 input_seed=synth.INPUT_SEED, oracle_sha256=oracle_hash(), variant=v)
        print(f"wrote {golden_path(a.workload, v)}  min margin {margin.min():.3e}", flush=True)


if __name__ == "__main__":
    main()
