#!/usr/bin/env python3
"""Benchmark of the decoder hot path on one MI355X.

One "step" = one whole pass of the hot path over one synthetic request of the
configuration the metric is quoted on (Qwen3-0.6B-shaped, bf16 weights and KV cache,
fp32 accumulation, batch 1): reset the KV slot, run the 128-token prompt, then 128
greedy decode steps with the token fed back on the device.  The paper's metric is
tokens/s over the decoding stage (Section 4, experimental setup); `value` is that,
summed over the K timed steps, with weights and prompt already resident in HBM.
--workload selects the larger configurations (batched requests fill every slot's
context with prompt passes, then decode all slots together).

Prints ONE JSON line.  `roofline`: algorithmic bytes of the decode launches (every weight
element and every cached K/V element once per step) over their duration, against the
published HBM peak, plus the HBM traffic measured with counters where a summary for the
workload is committed.  `cpu_baseline`: the fp64 CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix cores, published
WORKLOADS = {
    # name: (shape key, batch, context tokens filled by the prompt pass per slot, decode steps)
    "qwen3-0.6b-bf16-b1-p128-d128": ("qwen3-0.6b", 1, 128, 128),
    "qwen3-1.7b-bf16-b1-p512-d256": ("qwen3-1.7b", 1, 512, 256),
    "qwen3-4b-bf16-b1-c2048-d128": ("qwen3-4b", 1, 2048, 128),
    "qwen3-4b-bf16-b8-c2048-d128": ("qwen3-4b", 8, 2048, 128),
    "qwen3-8b-bf16-b16-c4096-d128": ("qwen3-8b", 16, 4096, 128),
}


def algorithmic_bytes_per_decode_step(shape, ctx_mean: float, batch: int = 1) -> float:
    """Every weight element once per step, every cached K/V element of every sequence once per step."""
    w = 2 if shape.dtype == 1 else 4
    per_layer = (shape.dq + 2 * shape.dkv) * shape.hidden + shape.hidden * shape.dq + 3 * shape.ffn * shape.hidden
    weights = w * (shape.n_layers * per_layer + shape.vocab * shape.hidden)
    kv = shape.n_layers * 2 * shape.dkv * w * ctx_mean * batch
    return float(weights + kv)


def counter_traffic(workload: str, decode_steps: int):
    """HBM bytes per launch of the resident kernel as measured with rocprofv3 counters
    (FETCH_SIZE + WRITE_SIZE, scaled by a known copy); read from the committed summary of
    that measurement, which is valid for the same workload only.  None if there is none."""
    pdir = os.path.join(ROOT, "profiles")
    try:
        names = sorted(n for n in os.listdir(pdir) if n.endswith("__hbm_traffic.txt"))
    except OSError:
        return None
    for name in names:
        for line in open(os.path.join(pdir, name)):
            if line.startswith("traffic_bytes_per_launch="):
                kv = dict(f.split("=") for f in line.split())
                if kv.get("workload") == workload and int(kv.get("decode_steps", -1)) == decode_steps:
                    return int(kv["traffic_bytes_per_launch"])
    return None


def resident_stage_trace(model, nnc, shape, prompt):
    """Per-stage times of one decode step inside the resident kernel: every workgroup stamps the
    100 MHz wall clock at its stage boundaries; mean / fastest / slowest workgroup of the
    per-layer means, in microseconds."""
    import numpy as np
    model.kv_reset(0)
    _, nxt = model.prefill(0, prompt, want_logits=False)
    first = int(nxt.item())
    model.decode_greedy([0], [first], 8)
    model.set_option(nnc.OPT_STAGE_TRACE, 5 + 1)               # trace step 5 of the next launch
    model.decode_greedy([0], [first], 16)
    model.synchronize()
    t = model.stage_trace().astype(np.int64)
    model.set_option(nnc.OPT_STAGE_TRACE, 0)
    L = shape.n_layers
    names = ["wait for x + input norm", "QKV GEMM + publish", "attention", "merge + O projection",
             "wait for x + post-attention norm", "gate|up GEMM + publish", "down projection", "to next layer"]
    per = t[:, :8 * L].reshape(-1, L, 8)
    nxt_start = np.concatenate([per[:, 1:, 0], t[:, 8 * L:8 * L + 1]], axis=1)
    d = np.diff(np.concatenate([per, nxt_start[:, :, None]], axis=2), axis=2) * 0.01
    lo = min(2, L - 1)                                          # skip the first layers of the step (cold prefetch)
    out = {"per_layer": [{"stage": n, "mean": round(float(d[:, lo:, i].mean()), 2),
                          "fastest_wg": round(float(d[:, lo:, i].mean(axis=1).min()), 2),
                          "slowest_wg": round(float(d[:, lo:, i].mean(axis=1).max()), 2)}
                         for i, n in enumerate(names)],
           "layer_total": round(float(d[:, lo:, :].sum(axis=2).mean()), 2)}
    fin = np.diff(t[:, 8 * L - 1:], axis=1) * 0.01
    out["after_last_layer"] = {"wait + final norm": round(float(fin[:, 0].mean()), 2),
                               "LM head": round(float(fin[:, 1].mean()), 2),
                               "token exchange": round(float(fin[:, 2].mean()), 2)}
    out["step_total"] = round(float((t[0, -1] - t[0, 0]) * 0.01), 2)
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="qwen3-0.6b-bf16-b1-p128-d128", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget for the oracle timing sample")
    ap.add_argument("--stage-trace", action="store_true",
                    help="batch-1 workloads: add the resident decode kernel's per-stage wall-clock times of one step")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no cross-GPU sharding or collectives); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import synth
    from paper_2512_21571_amd import binding as nnc

    shape_key, B, T, S = WORKLOADS[args.workload]
    shape = synth.SHAPES[shape_key]
    blob = synth.make_blob(shape)
    model = nnc.Model(shape, blob, B, T + S)
    prompts = [synth.tokens(T, shape.vocab, stream=b) for b in range(B)]
    prompt = prompts[0]
    slots = list(range(B))
    stream = model.stream

    def one_pass(events=None):
        model.kv_reset(-1)
        if events:
            events[0].record(stream)
        nxt = [model.prefill(b, prompts[b], want_logits=False)[1] for b in slots]
        if events:
            events[1].record(stream)
        firsts = [int(t.item()) for t in nxt]       # the one host round trip of a request
        if events:
            events[2].record(stream)
        toks, _ = model.decode_greedy(slots, firsts, S)
        if events:
            events[3].record(stream)
        return toks

    for _ in range(args.warmup):
        one_pass()
    torch.cuda.synchronize()

    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        toks = one_pass(evs[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    prefill_ms = sum(e[0].elapsed_time(e[1]) for e in evs)
    decode_ms = sum(e[2].elapsed_time(e[3]) for e in evs)
    decode_tok_s = args.steps * S * B / (decode_ms * 1e-3)
    prefill_tok_s = args.steps * T * B / (prefill_ms * 1e-3)
    ctx_mean = T + (S - 1) / 2.0 + 1
    step_bytes = algorithmic_bytes_per_decode_step(shape, ctx_mean, B)
    decode_ms_per_token = decode_ms / (args.steps * S)   # per decode step (B tokens)

    # The dominant kernel: at batch 1 the resident decode kernel runs all S steps of a request
    # in one launch, so the HIP events around nnc_decode_greedy (recorded on the stream the
    # kernel is launched on) bracket exactly that launch plus one 512-byte copy of the token
    # log.  Algorithmic bytes per launch = S decode steps x bytes per step (weights once per
    # step, cached K/V rows once per step).  At batch > 1 the same events bracket S replays of
    # the captured per-stage graph, reported as one unit.
    launch_ms = decode_ms / args.steps
    launch_bytes = step_bytes * S
    achieved = launch_bytes / (launch_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "k_decode_resident" if B == 1 else "decode step graph (per-stage kernels)",
                "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": counter_traffic(args.workload, S),
                "launches": args.steps, "avg_launch_us": round(launch_ms * 1e3, 1),
                "bytes_per_launch": round(launch_bytes)}

    # per-kernel durations of the per-stage path (prompt pass and its kernels): the same request
    # again with every launch bracketed by HIP events inside the library
    model.kv_reset(0)
    model.profile_begin()
    model.prefill(0, prompt, want_logits=False)
    stats = model.profile_end()
    gemm = [r for r in stats if r["name"] == "gemm_prefill" and r["total_ms"] > 0]
    prefill_gemm_tflops = gemm[0]["flops"] / (gemm[0]["total_ms"] * 1e-3) / 1e12 if gemm else None

    # one plain device-to-device copy of known size (1 GiB read + 1 GiB written), untimed: the
    # reference a counter run (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) scales its readings by
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst

    stage_trace = None
    if args.stage_trace and B == 1:
        stage_trace = resident_stage_trace(model, nnc, shape, prompt)

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        o = oracle.from_shape(shape, blob, 1, 16 + S)
        ctx0 = 16                                    # short prompt so the sample is mostly decode
        _, t = o.prefill(0, prompt[:ctx0], oracle.ROUND_KV)
        n, c0 = 0, time.perf_counter()
        while n < S and time.perf_counter() - c0 < args.cpu_seconds:
            _, t = o.step_token(0, t, oracle.ROUND_KV)
            n += 1
        dt = time.perf_counter() - c0
        cpu = {"value": round(n / dt, 3), "unit": "tokens/s", "cores": oracle.get_threads(), "kind": "oracle",
               "sample": f"{n} greedy decode steps of the same model after a {ctx0}-token prompt, fp64, "
                         f"{oracle.get_threads()} OpenMP threads"}

    out = {
        "metric": "decode tokens/s + achieved HBM GB/s fraction; prefill tokens/s + MFMA util",
        "value": round(decode_tok_s, 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(wall * 1e3 / args.steps, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "batch": B, "prompt_tokens": T, "decode_steps": S,
                   "weights": "N(0,0.02) seeded, bf16", "kv_cache": "bf16"},
        "decode_ms_per_token": round(decode_ms_per_token, 5),
        "decode_hbm_frac_step": round(step_bytes / (decode_ms_per_token * 1e-3) / (HBM_PEAK_GBS * 1e9), 4),
        "decode_algorithmic_bytes_per_step": round(step_bytes),
        "prefill_tokens_per_s": round(prefill_tok_s, 1),
        "prefill_ms": round(prefill_ms / args.steps, 4),
        "prefill_gemm_tflops": round(prefill_gemm_tflops, 1) if prefill_gemm_tflops else None,
        "prefill_gemm_mfma_frac": round(prefill_gemm_tflops / MFMA_BF16_PEAK_TFLOPS, 4) if prefill_gemm_tflops else None,
        "roofline": roofline,
        "prefill_kernels": [{"name": r["name"], "launches": r["launches"], "total_ms": round(r["total_ms"], 4)}
                            for r in stats],
        "cpu_baseline": cpu,
    }
    if stage_trace is not None:
        out["decode_stage_trace_us"] = stage_trace
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
