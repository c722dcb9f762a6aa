#!/usr/bin/env python3
"""Benchmark of the decoder hot path on one MI355X.

One "step" = one whole pass of the hot path over one batch of synthetic requests.  The default
workload is the largest single-GPU configuration (Qwen3-8B-shaped, bf16 weights and KV cache,
fp32 accumulation, 16 sequences): reset the KV slots, run a 4096-token prompt pass per slot
(2048-token matrix-core blocks), read the 16 first tokens back, then 128 greedy decode steps of
all 16 sequences with the tokens fed back on the device.  The paper's metric is tokens/s over
the decoding stage (Section 4, experimental setup); `value` is that, summed over the K timed
steps, with weights and prompts already resident in HBM.  --workload selects the other
configurations (the batch-1 ones decode inside one resident kernel launch per request).

Prints ONE JSON line.  `roofline`: the dominant decode kernel (by summed time), its algorithmic
bytes per launch (every weight element of its matrix once) over its average launch duration,
measured with HIP events on the model's stream, against the published HBM peak, plus the HBM
traffic per launch measured with counters where a summary for the workload is committed.
`roofline_prefill_gemm`: the same for the prompt GEMM kernel against the bf16 matrix-core peak.
`cpu_baseline`: the fp64 CPU oracle timed on a bounded sample.  `parity`: a short leg that
compares logits with the oracle (live for the small models, against the committed full-depth
expected values of the oracle for the 4B / 8B workloads).
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
    "qwen3-0.6b-f16-b1-p128-d128": ("qwen3-0.6b-f16", 1, 128, 128),
    "qwen3-1.7b-bf16-b1-p512-d256": ("qwen3-1.7b", 1, 512, 256),
    "qwen3-4b-bf16-b1-c2048-d128": ("qwen3-4b", 1, 2048, 128),
    "qwen3-4b-bf16-b8-c2048-d128": ("qwen3-4b", 8, 2048, 128),
    "qwen3-8b-bf16-b16-c4096-d128": ("qwen3-8b", 16, 4096, 128),
    # weight-only 8-bit layers (bytes + one scale per output row), bf16 activations / cache / LM head
    "qwen3-8b-w8-b16-c512-d128": ("qwen3-8b-w8", 16, 512, 128),
    "qwen3-8b-w8-b16-c4096-d128": ("qwen3-8b-w8", 16, 4096, 128),
    "qwen3-8b-bf16-b16-c512-d128": ("qwen3-8b", 16, 512, 128),
}


def algorithmic_bytes_per_decode_step(shape, ctx_mean: float, batch: int = 1) -> float:
    """Every weight element once per step, every cached K/V element of every sequence once per step."""
    w = 4 if shape.dtype == 0 else 2
    lw = 1 if shape.dtype == 3 else w                       # weight-only 8-bit layers (their scales: 4 bytes per row)
    per_layer = (shape.dq + 2 * shape.dkv) * shape.hidden + shape.hidden * shape.dq + 3 * shape.ffn * shape.hidden
    scales = 4 * (shape.dq + 2 * shape.dkv + 2 * shape.hidden + 2 * shape.ffn) if shape.dtype == 3 else 0
    weights = shape.n_layers * (lw * per_layer + scales) + w * shape.vocab * shape.hidden
    kv = shape.n_layers * 2 * shape.dkv * w * ctx_mean * batch
    return float(weights + kv)


def counter_traffic(workload: str, kernel: str, decode_steps: int):
    """Mean HBM bytes per launch of `kernel` as measured with rocprofv3 counters (FETCH_SIZE +
    WRITE_SIZE, each scaled by what it reads for a known copy); taken from the committed summary
    of that measurement, which is valid for the same workload and kernel only.  None if there
    is none."""
    pdir = os.path.join(ROOT, "profiles")
    try:
        names = sorted(n for n in os.listdir(pdir) if n.endswith("__hbm_traffic.txt"))
    except OSError:
        return None
    for name in names:
        for line in open(os.path.join(pdir, name)):
            if line.startswith("traffic_bytes_per_launch="):
                kv = dict(f.split("=") for f in line.split())
                if (kv.get("workload") == workload and kv.get("kernel", "k_decode_resident") == kernel
                        and int(kv.get("decode_steps", decode_steps)) == decode_steps):
                    return int(kv["traffic_bytes_per_launch"])
    return None


# the block-tile prompt GEMM: the 256 x 256 tile kernel (k_gemm_prefill_big) or the 256 / 192 / 128 x 128 one
# (k_gemm_prefill_dl), chosen per launch by the library's tile chooser; timed together as one family
PG_KERNELS = "k_gemm_prefill_big|k_gemm_prefill_dl"
KERNEL_OF_FAMILY = {"gemm_skinny": "k_gemm_skinny", "attn_partial": "k_attn_partial_mc",
                    "rmsnorm_pack": "k_rmsnorm_pack", "attn_combine": "k_attn_combine",
                    "gemm_prefill": PG_KERNELS, "attn_prefill": "k_attn_prefill"}
GOLDEN = {"qwen3-4b-bf16-b1-c2048-d128": "cfg3", "qwen3-4b-bf16-b8-c2048-d128": "cfg3",
          "qwen3-8b-bf16-b16-c4096-d128": "cfg4"}


def by_kernel(stats):
    """Per-kernel records from the library's per-family ones (the skinny GEMM reports one family
    per matrix it streams: added up here, kept separately as `parts`)."""
    out = {}
    for r in stats:
        fam = r["name"]
        k = KERNEL_OF_FAMILY.get(fam.split(".")[0], fam)
        d = out.setdefault(k, {"name": k, "launches": 0, "total_ms": 0.0, "bytes": 0.0, "flops": 0.0, "parts": {}})
        for f in ("launches", "total_ms", "bytes", "flops"):
            d[f] += r[f]
        if "." in fam and r["total_ms"] > 0:
            d["parts"][fam.split(".", 1)[1]] = {"launches": r["launches"],
                                                 "avg_us": round(r["total_ms"] * 1e3 / r["launches"], 2),
                                                 "GBps": round(r["bytes"] / (r["total_ms"] * 1e-3) / 1e9, 1),
                                                 "TFLOPs": round(r["flops"] / (r["total_ms"] * 1e-3) / 1e12, 1)}
    return list(out.values())


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


def percentile(v, q):
    v = sorted(v)
    return v[min(len(v) - 1, int(round(q * (len(v) - 1))))]


def compare(model, prompt, want, others=()):
    """GPU logits of slot 0's prompt pass and of decode steps teacher-forced on the expected
    tokens against `want` = [(fp64 logits, greedy token)]: max abs error, agreement, margin.
    `others`: prompts of slots 1 ..; with them slot 0 decodes as column 0 of the full batch (the
    timed launch configuration), the other slots following their own greedy tokens."""
    import numpy as np
    model.kv_reset(-1)
    lg, _ = model.prefill(0, prompt)
    got = [lg.double().cpu().numpy()]
    slots = list(range(1 + len(others)))
    rest = [int(model.prefill(b + 1, p, want_logits=False)[1].item()) for b, p in enumerate(others)]
    for i in range(len(want) - 1):
        lg, nx = model.decode_step(slots, [want[i][1]] + rest)
        got.append(lg[0].double().cpu().numpy())
        rest = [int(v) for v in nx.tolist()[1:]]
    err, agree, margin, flips = 0.0, 0, float("inf"), []
    for i, (g, (lo, t)) in enumerate(zip(got, want)):
        e = float(np.abs(g - lo).max())
        err = max(err, e)
        part = np.partition(lo, -2)
        mg = float(part[-1] - part[-2])
        margin = min(margin, mg)
        if int(np.argmax(g)) == t:
            agree += 1
        else:
            # a different arg-max where the oracle's own top two are closer than twice the error at
            # that position is a tie within the error, not a wrong token
            flips.append({"position": i, "oracle_top2_margin": round(mg, 6), "abs_err": round(e, 6),
                          "tie_within_error": mg <= 2.0 * e})
    out = {"positions": len(want), "batch": len(slots), "max_abs_err": round(err, 6),
           "greedy_agreement": round(agree / len(want), 4), "min_margin": round(margin, 6)}
    if flips:
        out["disagreements"] = flips
    return out


def parity_full_depth(model, workload, prompt, others=()):
    """Slot 0 at the workload's full context against the expected values the oracle wrote offline
    (tests/golden/, full depth; prompt blocks mirrored); None where no such file is committed."""
    import numpy as np
    gold = GOLDEN.get(workload)
    path = os.path.join(ROOT, "tests", "golden", f"{gold}_slot0_mirrored.npz") if gold else None
    if not path or not os.path.exists(path):
        return None
    z = np.load(path)
    want = [(z["logits"][i].astype(np.float64), int(z["next"][i])) for i in range(len(z["next"]))]
    out = compare(model, prompt, want, others)
    out["reference"] = ("full-depth oracle values written offline (prompt rounding points mirrored), full context; "
                        "slot 0 decoded as one column of the workload's batch")
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="qwen3-8b-bf16-b16-c4096-d128", choices=sorted(WORKLOADS))
    ap.add_argument("--decode-steps", type=int, default=0,
                    help="decode steps per request instead of the workload's (short profiler runs)")
    ap.add_argument("--prefill-block", type=int, default=0,
                    help="tokens per block of the prompt pass (NNC_OPT_PREFILL_BLOCK; 0 = the library's default)")
    ap.add_argument("--prefill-tile", type=int, default=-1, help="force a block tile of the prompt GEMMs (NNC_OPT_PREFILL_TILE)")
    ap.add_argument("--planner", type=int, default=1, help="0: the hand rules instead of the analytic tile chooser (NNC_OPT_PLANNER)")
    ap.add_argument("--decode-pieces", type=int, default=0, help="pieces per activation in batched decode GEMMs (NNC_OPT_DECODE_PIECES; 0 = the library's default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-parity", action="store_true")
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

    def note(msg):                                   # progress on stderr; stdout carries the one JSON line
        print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)

    shape_key, B, T, S = WORKLOADS[args.workload]
    if args.decode_steps > 0:
        S = args.decode_steps
    shape = synth.SHAPES[shape_key]
    note(f"workload {args.workload}: generating the weight blob")
    blob = synth.make_blob(shape)
    note(f"blob {blob.nbytes / 1e9:.2f} GB; creating the model (upload + repack)")
    model = nnc.Model(shape, blob, B, T + S + 8)       # + the few extra steps of the per-kernel leg
    if args.prefill_block:
        model.set_option(nnc.OPT_PREFILL_BLOCK, args.prefill_block)
    if not args.planner:
        model.set_option(nnc.OPT_PLANNER, 0)
    if args.prefill_tile >= 0:
        model.set_option(nnc.OPT_PREFILL_TILE, args.prefill_tile)
    if args.decode_pieces:
        model.set_option(nnc.OPT_DECODE_PIECES, args.decode_pieces)
    note("model ready; warm-up passes")
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
        return toks, firsts

    for _ in range(args.warmup):
        one_pass()
    torch.cuda.synchronize()
    note(f"timing {args.steps} passes")

    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        toks, firsts = one_pass(evs[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    prefill_ms = sum(e[0].elapsed_time(e[1]) for e in evs)
    decode_ms = sum(e[2].elapsed_time(e[3]) for e in evs)
    decode_tok_s = args.steps * S * B / (decode_ms * 1e-3)
    prefill_tok_s = args.steps * T * B / (prefill_ms * 1e-3)
    ctx_mean = T + (S - 1) / 2.0 + 1
    step_bytes = algorithmic_bytes_per_decode_step(shape, ctx_mean, B)
    decode_ms_per_token = decode_ms / (args.steps * S)   # per decode step (B tokens)

    # per-step latency of the single-step entry point (one call per step, events between calls):
    # p50 / p99 over the S steps that follow the timed passes' prompt state
    note("timed passes done; per-step latency leg")
    toks_host = toks.cpu().numpy()
    model.kv_reset(-1)
    firsts = [int(model.prefill(b, prompts[b], want_logits=False)[1].item()) for b in slots]
    lat_ev = [torch.cuda.Event(enable_timing=True) for _ in range(S + 1)]
    cur = firsts
    lat_ev[0].record(stream)
    nxt_dev = None
    for i in range(S):
        _, nxt_dev = model.decode_step(slots, cur, want_logits=False)
        lat_ev[i + 1].record(stream)
        cur = [int(v) for v in toks_host[i]]         # the tokens the greedy loop produced (same state)
    torch.cuda.synchronize()
    lat = [lat_ev[i].elapsed_time(lat_ev[i + 1]) for i in range(S)]
    step_latency = {"p50": round(percentile(lat, 0.5), 4), "p99": round(percentile(lat, 0.99), 4),
                    "mean": round(sum(lat) / len(lat), 4), "unit": "ms",
                    "what": "nnc_decode_step, one call per step, tokens passed from the host"}

    # The dominant decode kernel.  Batch 1: the resident kernel runs all S steps of a request in
    # one launch, bracketed by the events around nnc_decode_greedy (recorded on the stream the
    # kernel is launched on); algorithmic bytes per launch = S x bytes per step.  Batch > 1: a
    # step is a graph of per-stage kernels; a few more steps run eagerly with every launch
    # bracketed by HIP events inside the library (same kernels, same arguments), the kernel with
    # the largest summed time is reported with its own algorithmic bytes (every weight element
    # of the launched matrix once) and its own mean duration.
    note("per-kernel event legs")
    decode_kernels = None
    if B == 1:
        launch_ms = decode_ms / args.steps
        launch_bytes = step_bytes * S
        achieved = launch_bytes / (launch_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "k_decode_resident", "achieved": round(achieved, 1),
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "traffic": counter_traffic(args.workload, "k_decode_resident", S),
                    "launches": args.steps, "avg_launch_us": round(launch_ms * 1e3, 1),
                    "bytes_per_launch": round(launch_bytes)}
    else:
        model.profile_begin()
        model.decode_greedy(slots, cur, 4)
        dstats = by_kernel(model.profile_end())
        decode_kernels = [{"name": r["name"], "launches": r["launches"], "total_ms": round(r["total_ms"], 4),
                           "algorithmic_GBps": round(r["bytes"] / (r["total_ms"] * 1e-3) / 1e9, 1) if r["total_ms"] > 0 else None,
                           **({"parts": r["parts"]} if r["parts"] else {})}
                          for r in dstats]
        dom = max(dstats, key=lambda r: r["total_ms"])
        kname = dom["name"]
        achieved = dom["bytes"] / (dom["total_ms"] * 1e-3) / 1e9
        # An event pair brackets launch to launch: in these eager steps that includes the time
        # between one kernel's end and the next one's start, which the captured graph of the timed
        # region mostly hides.  Its size per launch: (eager step - timed step) / launches per step.
        # Reported beside the raw figure (a kernel trace's start-to-end durations correspond to
        # the figure without it); `achieved` stays the raw, lower one.
        n_launch_step = sum(r["launches"] for r in dstats) / 4.0
        eager_step_ms = sum(r["total_ms"] for r in dstats) / 4.0
        timed_step_ms = decode_ms / args.steps / S
        gap_us = max(0.0, (eager_step_ms - timed_step_ms) * 1e3 / n_launch_step)
        avg_us = dom["total_ms"] * 1e3 / dom["launches"]
        roofline = {"bound": "hbm", "kernel": kname, "achieved": round(achieved, 1),
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "traffic": counter_traffic(args.workload, kname, S),
                    "launches": dom["launches"], "avg_launch_us": round(avg_us, 2),
                    "bytes_per_launch": round(dom["bytes"] / dom["launches"]),
                    "eager_launch_gap_us": round(gap_us, 2),
                    "achieved_without_launch_gap": round(dom["bytes"] / dom["launches"] / ((avg_us - gap_us) * 1e-6) / 1e9, 1)
                    if avg_us > gap_us else None}

    # per-kernel durations of the prompt pass: the same request again with every launch
    # bracketed by HIP events inside the library
    model.kv_reset(0)
    model.profile_begin()
    model.prefill(0, prompt, want_logits=False)
    stats = by_kernel(model.profile_end())
    gemm = [r for r in stats if r["name"] == PG_KERNELS and r["total_ms"] > 0]
    prefill_gemm_tflops = gemm[0]["flops"] / (gemm[0]["total_ms"] * 1e-3) / 1e12 if gemm else None
    roofline_pg = None
    if gemm:
        roofline_pg = {"bound": "mfma", "kernel": PG_KERNELS, "achieved": round(prefill_gemm_tflops, 1),
                       "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                       "frac": round(prefill_gemm_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                       "traffic": counter_traffic(args.workload, PG_KERNELS, S),
                       "launches": gemm[0]["launches"],
                       "avg_launch_us": round(gemm[0]["total_ms"] * 1e3 / gemm[0]["launches"], 2),
                       "flops_per_launch": round(gemm[0]["flops"] / gemm[0]["launches"])}

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

    note("parity and oracle legs")
    parity = None if args.no_parity else parity_full_depth(model, args.workload, prompt, prompts[1:])

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        ofl = oracle.ROUND_KV | (oracle.ROUND_F16 if shape.dtype == 2 else 0)   # the 16-bit cache, in the model's format
        o = oracle.from_shape(shape, blob, 1, 16 + S + 8)    # + the one-thread sample's steps
        ctx0 = 16                                    # short prompt so the sample is mostly decode
        lo, t = o.prefill(0, prompt[:ctx0], ofl)
        want = [(lo, t)]
        n, c0 = 0, time.perf_counter()
        while n < S and time.perf_counter() - c0 < args.cpu_seconds:
            lo, t = o.step_token(0, t, ofl)
            want.append((lo, t))
            n += 1
        dt = time.perf_counter() - c0
        cpu = {"value": round(n / dt, 3), "unit": "tokens/s", "cores": oracle.get_threads(), "kind": "oracle",
               "sample": f"{n} greedy decode steps of one sequence of the same model after a {ctx0}-token prompt "
                         f"(the workload's context is {T}: cached rows add {100.0 * shape.n_layers * 2 * shape.dq * T / (sum_macs(shape)):.0f} % "
                         f"to the multiply-adds of a step), fp64, {oracle.get_threads()} OpenMP threads"}
        if not args.no_parity:
            # the oracle run just timed doubles as a reference: the same short request on the GPU
            cpu["parity_of_the_sample"] = compare(model, prompt[:ctx0], want)
        if B == 1 and shape.hidden <= 2048:
            # the paper's single-thread rows (Section 4.1) have a counterpart: the oracle on one thread
            threads = oracle.get_threads()
            oracle.set_threads(1)
            n1, c1 = 0, time.perf_counter()
            while n1 < 8 and time.perf_counter() - c1 < args.cpu_seconds / 2:
                _, t = o.step_token(0, t, ofl)
                n1 += 1
            cpu["one_thread_tokens_per_s"] = round(n1 / (time.perf_counter() - c1), 3)
            oracle.set_threads(threads)

    dname = {0: "f32", 1: "bf16", 2: "f16", 3: "bf16"}[shape.dtype]   # byte weights compute in bf16
    out = {
        "metric": "decode tokens/s + achieved HBM GB/s fraction; prefill tokens/s + MFMA util",
        "value": round(decode_tok_s, 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(wall * 1e3 / args.steps, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": dname, "data": "synthetic",
        "config": {"workload": args.workload, "batch": B, "prompt_tokens": T, "decode_steps": S,
                   "weights": "N(0,0.02) seeded, " + ("8-bit with per-row scales (layers), bf16 (embedding, LM head)"
                                                      if shape.dtype == 3 else dname), "kv_cache": dname},
        "decode_ms_per_token": round(decode_ms_per_token, 5),
        "decode_hbm_frac_step": round(step_bytes / (decode_ms_per_token * 1e-3) / (HBM_PEAK_GBS * 1e9), 4),
        "decode_algorithmic_bytes_per_step": round(step_bytes),
        "decode_step_latency_ms": step_latency,
        "prefill_tokens_per_s": round(prefill_tok_s, 1),
        "prefill_ms": round(prefill_ms / args.steps, 4),
        "prefill_gemm_tflops": round(prefill_gemm_tflops, 1) if prefill_gemm_tflops else None,
        "prefill_gemm_mfma_frac": round(prefill_gemm_tflops / MFMA_BF16_PEAK_TFLOPS, 4) if prefill_gemm_tflops else None,
        "roofline": roofline,
        "roofline_prefill_gemm": roofline_pg,
        "decode_kernels": decode_kernels,
        "prefill_kernels": [{"name": r["name"], "launches": r["launches"], "total_ms": round(r["total_ms"], 4),
                             **({"parts": r["parts"]} if r["parts"] else {})} for r in stats],
        "parity": parity,
        "cpu_baseline": cpu,
    }
    if stage_trace is not None:
        out["decode_stage_trace_us"] = stage_trace
    print(json.dumps(out))
    return 0


def sum_macs(shape) -> float:
    per_layer = (shape.dq + 2 * shape.dkv) * shape.hidden + shape.hidden * shape.dq + 3 * shape.ffn * shape.hidden
    return float(shape.n_layers * per_layer + shape.vocab * shape.hidden)


if __name__ == "__main__":
    sys.exit(main())
