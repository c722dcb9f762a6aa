"""GPU parity at the benchmark configurations' full sizes.

config 0: one Qwen3-0.6B-shaped layer, fp32, 16-token prompt + 16 decode steps,
          hidden states compared row by row, infinity-norm relative error <= 1e-4.
config 1: full Qwen3-0.6B-shaped model, bf16 weights and KV cache, fp32 accumulation,
          128-token prompt (large-block matrix-core path, two bf16 pieces per GEMM input)
          + 128 greedy steps: max abs logit error <= 3e-2 at the prompt's
          last position and at every decode step (teacher-forced on the oracle's tokens),
          greedy tokens equal at every step, and the free-running on-device greedy loop
          (the launch configuration bench.py times) reproduces the oracle's tokens.
config 2: full Qwen3-1.7B-shaped model, 512-token prompt + all 256 decode steps, the same way.
configs 3, 4 (4B / 8B shapes): (i) real layer shape, vocabulary, context and batch with the depth
          cut to 2 / 1 layers so that the live oracle can follow every slot; (ii) full depth,
          short contexts, live oracle on two slots of a full batch; (iii) full depth and full
          context against values the oracle wrote offline (tests/golden/); (iv) full-depth
          batch-invariance and replay checks.
A step whose oracle top-2 margin is below 4x that step's measured max error is a
"tie within error": it is counted and printed, only such a step may disagree, and the
fixed-seed runs here must have none.
"""
import hashlib
import os

import numpy as np
import pytest

import oracle
import synth
from parity_util import oracle_flags, oracle_prefill_like_library, rel_inf, top2_margin

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nnc():
    from paper_2512_21571_amd import binding
    binding.lib()
    return binding


def test_config0_one_layer_fp32(nnc):
    print("case: config 0 (one 0.6B-shaped layer, fp32)", flush=True)
    shape = synth.SHAPES["layer-0.6b-f32"]
    blob = synth.make_blob(shape)
    g = nnc.Model(shape, blob, 1, 32)
    o = oracle.from_shape(shape, blob, 1, 32)
    x = synth.activations(32, shape.hidden)
    want = np.stack([o.step_hidden(0, x[t].astype(np.float64)) for t in range(32)])
    got = [g.prefill_hidden(0, x[:16]).double().cpu().numpy()]
    for t in range(16, 32):
        got.append(g.decode_step_hidden([0], x[t:t + 1]).double().cpu().numpy())
    got = np.concatenate(got)
    errs = [rel_inf(got[t], want[t]) for t in range(32)]
    print(f"config0 max rel-inf error {max(errs):.3e}", flush=True)
    assert max(errs) <= 1e-4


def test_config1_qwen3_0p6b_bf16_prompt128_decode128(nnc):
    print("case: config 1 (0.6B-shaped, bf16, 128 + 128)", flush=True)
    shape = synth.SHAPES["qwen3-0.6b"]
    T, S = 128, 128
    blob = synth.make_blob(shape)
    g = nnc.Model(shape, blob, 1, T + S)
    o = oracle.from_shape(shape, blob, 1, T + S)
    fl = oracle_flags(shape)
    toks = synth.tokens(T, shape.vocab)

    # prompt pass: 128 tokens run on the large-block path with two bf16 pieces per GEMM input
    # (fp32-grade), so the oracle runs unrounded activations
    lo, first = o.prefill(0, toks, fl)
    lg, ng = g.prefill(0, toks)
    err = np.abs(lg.double().cpu().numpy() - lo).max()
    print(f"prompt last-position max abs err {err:.3e}, margin {top2_margin(lo):.3e}", flush=True)
    assert err <= 3e-2 and int(ng.item()) == first

    want_tokens, ties, max_err, min_margin = [], [], 0.0, np.inf
    t = first
    for step in range(S):
        lo, nxt = o.step_token(0, t, fl)
        lg, ng = g.decode_step([0], [t])
        e = np.abs(lg[0].double().cpu().numpy() - lo).max()
        mg = top2_margin(lo)
        max_err, min_margin = max(max_err, e), min(min_margin, mg)
        assert e <= 3e-2, (step, e)
        if int(ng.item()) != nxt:
            assert mg < 4 * e, (step, mg, e)
            ties.append(step)
        want_tokens.append(nxt)
        t = nxt
        if step % 32 == 31:
            print(f"  step {step + 1}: max abs err so far {max_err:.3e}, min margin {min_margin:.3e}", flush=True)
    print(f"decode max abs err {max_err:.3e}; min top-2 margin {min_margin:.3e}; ties within error: {ties}",
          flush=True)
    agree = 1.0 - len(ties) / S
    assert agree == 1.0, f"greedy agreement {agree:.4f}, tie steps {ties}"

    # free-running greedy loop on the device (graph replay), as timed by the benchmark
    g.kv_reset(0)
    g.prefill(0, toks, want_logits=False)
    got, _ = g.decode_greedy([0], [first], S)
    got = got.cpu().numpy()[:, 0]
    assert np.array_equal(got, np.array(want_tokens))


def _check_step(lg_row, lo, label, stats):
    """One position: max abs logit error <= 3e-2; the greedy tokens agree unless the oracle's
    top-2 margin is within 4x the measured error of that position (a tie within error)."""
    got = lg_row.double().cpu().numpy()
    assert np.isfinite(got).all(), label
    e = float(np.abs(got - lo).max())
    mg = top2_margin(lo)
    stats["err"] = max(stats["err"], e)
    stats["margin"] = min(stats["margin"], mg)
    assert e <= stats.get("bar", 3e-2), (label, e)
    if int(np.argmax(got)) != int(np.argmax(lo)):
        assert mg < 4 * e, (label, mg, e)
        stats["ties"].append(label)


def test_config2_qwen3_1p7b_bf16_prompt512_decode(nnc):
    print("case: config 2 (1.7B-shaped, bf16, prompt 512, decode)", flush=True)
    shape = synth.SHAPES["qwen3-1.7b"]
    T, S, S_ORACLE = 512, 256, 256
    blob = synth.make_blob(shape)
    g = nnc.Model(shape, blob, 1, T + S)
    o = oracle.from_shape(shape, blob, 1, T + S)
    fl = oracle_flags(shape)
    toks = synth.tokens(T, shape.vocab)
    stats = dict(err=0.0, margin=np.inf, ties=[])
    lo, first = o.prefill(0, toks, fl)                      # 512 tokens: two bf16 pieces per GEMM input
    lg, ng = g.prefill(0, toks)
    _check_step(lg, lo, "prompt", stats)
    print(f"  prompt: max abs err {stats['err']:.3e}, margin {stats['margin']:.3e}", flush=True)
    # all S decode steps against the oracle, teacher-forced on the oracle's tokens
    want, t = [], first
    for step in range(S_ORACLE):
        lo, nxt = o.step_token(0, t, fl)
        lg, _ = g.decode_step([0], [t])
        _check_step(lg[0], lo, f"step {step}", stats)
        want.append(nxt)
        t = nxt
        if step % 64 == 63:
            print(f"  step {step + 1}: max abs err so far {stats['err']:.3e}, min margin {stats['margin']:.3e}", flush=True)
    print(f"  {S_ORACLE} steps: max abs err {stats['err']:.3e}, min margin {stats['margin']:.3e}, "
          f"ties within error {stats['ties']}", flush=True)
    assert not stats["ties"]
    # the whole 256-step on-device greedy loop (the timed configuration) gives the oracle's
    # tokens, and a second run reproduces all 256 bit for bit
    g.kv_reset(0)
    g.prefill(0, toks, want_logits=False)
    a, _ = g.decode_greedy([0], [first], S)
    g.kv_reset(0)
    g.prefill(0, toks, want_logits=False)
    b, _ = g.decode_greedy([0], [first], S)
    a, b = a.cpu().numpy()[:, 0], b.cpu().numpy()[:, 0]
    assert np.array_equal(a[:S_ORACLE], np.array(want))
    assert np.array_equal(a, b)


def _sampled_depth(nnc, base, n_layers, long_ctx, batch, steps, label):
    """Configs 3 and 4 at their real layer shape, vocabulary and context, with the depth cut to
    what the fp64 oracle finishes in about a minute: slot 0 holds the full context (filled by the
    large-block prompt path, its single-bf16 blocks mirrored by the oracle), the other slots
    short ragged contexts; then batched decode steps, every slot compared with the oracle."""
    import dataclasses
    shape = dataclasses.replace(synth.SHAPES[base], name=f"{base}-{n_layers}layers", n_layers=n_layers)
    blob = synth.make_blob(shape)
    g = nnc.Model(shape, blob, batch, long_ctx + steps + 8)
    o = oracle.from_shape(shape, blob, batch, long_ctx + steps + 8)
    fl = oracle_flags(shape)
    stats = dict(err=0.0, margin=np.inf, ties=[])
    lens = [long_ctx] + [24 + 37 * i for i in range(1, batch)]
    t = []
    for b, n in enumerate(lens):
        toks = synth.tokens(n, shape.vocab, stream=b)
        lg, _ = g.prefill(b, toks)
        lo, nxt = oracle_prefill_like_library(o, b, toks, shape)
        _check_step(lg, lo, f"{label} prompt slot {b}", stats)
        t.append(nxt)
    print(f"  {label}: prompts max abs err {stats['err']:.3e}", flush=True)
    slots = list(range(batch))
    for step in range(steps):
        lg, _ = g.decode_step(slots, t)
        nxt = []
        for b in slots:
            lo, nb = o.step_token(b, t[b], fl)
            _check_step(lg[b], lo, f"{label} step {step} slot {b}", stats)
            nxt.append(nb)
        t = nxt
    # batch 1 on the long slot: the resident kernel with its merge stage
    for step in range(steps):
        lg, _ = g.decode_step([0], [t[0]])
        lo, t[0] = o.step_token(0, t[0], fl)
        _check_step(lg[0], lo, f"{label} b1 step {step}", stats)
    print(f"  {label}: max abs err {stats['err']:.3e}, min margin {stats['margin']:.3e}, ties {stats['ties']}", flush=True)
    assert not stats["ties"], stats["ties"]


def test_config3_qwen3_4b_shape_sampled_depth(nnc):
    print("case: config 3 layer shape (4B), 2 layers, context 2048, batch 8 and 1", flush=True)
    _sampled_depth(nnc, "qwen3-4b", 2, 2048, 8, 3, "cfg3")


def test_config4_qwen3_8b_shape_sampled_depth(nnc):
    print("case: config 4 layer shape (8B), 1 layer, context 4096, batch 16 and 1", flush=True)
    _sampled_depth(nnc, "qwen3-8b", 1, 4096, 16, 2, "cfg4")


_BIG = {}


def _big_model(nnc, name, batch, ctx):
    """The full-depth 4B / 8B models are expensive to generate and upload: one per module."""
    if name not in _BIG:
        shape = synth.SHAPES[name]
        blob = synth.make_blob(shape)
        _BIG[name] = (shape, blob, nnc.Model(shape, blob, batch, ctx + 24))
    shape, blob, g = _BIG[name]
    g.kv_reset(-1)
    return shape, blob, g


BIG = [("qwen3-4b", 8, 2048), ("qwen3-8b", 16, 4096)]


@pytest.mark.parametrize("name,batch,ctx", BIG)
def test_full_depth_batch_invariance(nnc, name, batch, ctx):
    """Configs 3 and 4 at full depth: the same sequence gives the same logits whether it is
    decoded alone or as one column of a full batch, and a replay of the greedy loop is
    bit-identical."""
    print(f"case: full-depth {name} batch {batch} context {ctx}", flush=True)
    shape, _, g = _big_model(nnc, name, batch, ctx)
    toks = synth.tokens(ctx, shape.vocab, stream=5)
    _, first = g.prefill(0, toks)
    first = int(first.item())
    short = [16 + 9 * b for b in range(1, batch)]
    firsts = [first]
    for b, n in enumerate(short, start=1):
        _, nx = g.prefill(b, synth.tokens(n, shape.vocab, stream=50 + b))
        firsts.append(int(nx.item()))
    slots = list(range(batch))
    lg_b, _ = g.decode_step(slots, firsts)            # slot 0 as a column of the batch
    row_b = lg_b[0].double().cpu().numpy()
    assert np.isfinite(lg_b.cpu().numpy()).all()
    # rewind slot 0 and decode it alone
    g.kv_reset(0)
    g.prefill(0, toks, want_logits=False)
    lg_1, _ = g.decode_step([0], [first])
    row_1 = lg_1[0].double().cpu().numpy()
    err = np.abs(row_b - row_1).max()
    print(f"  batch vs alone: max abs logit difference {err:.3e}, |logit| max {np.abs(row_1).max():.2f}", flush=True)
    assert err <= 3e-3
    # greedy loop replay on slot 0
    g.kv_reset(0)
    g.prefill(0, toks, want_logits=False)
    a, _ = g.decode_greedy([0], [first], 8)
    g.kv_reset(0)
    g.prefill(0, toks, want_logits=False)
    b, _ = g.decode_greedy([0], [first], 8)
    assert np.array_equal(a.cpu().numpy(), b.cpu().numpy())


@pytest.mark.parametrize("name,batch,ctx", BIG)
def test_full_depth_short_context_against_live_oracle(nnc, name, batch, ctx):
    """All 36 layers, every run: the first and the last slot of a full batch hold short prompts
    (two bf16 pieces per matrix-core input) and are followed by the oracle through the prompt
    pass and two batched decode steps; the other slots hold other short prompts.  Checks that
    nothing accumulates over the depth on the two-piece prompt path and the decode path."""
    print(f"case: full-depth {name}, short contexts, batch {batch}, oracle on slots 0 and {batch - 1}", flush=True)
    shape, blob, g = _big_model(nnc, name, batch, ctx)
    o = oracle.from_shape(shape, blob, 2, 64)
    fl = oracle_flags(shape)
    stats = dict(err=0.0, margin=np.inf, ties=[])
    lens = [40] + [11 + 3 * b for b in range(1, batch - 1)] + [17]
    watched = {0: 0, batch - 1: 1}                    # GPU slot -> oracle slot
    t = []
    for b, n in enumerate(lens):
        toks = synth.tokens(n, shape.vocab, stream=200 + b)
        lg, nx = g.prefill(b, toks)
        if b in watched:
            lo, no = o.prefill(watched[b], toks, fl)
            _check_step(lg, lo, f"prompt slot {b}", stats)
            t.append(no)
        else:
            t.append(int(nx.item()))
    print(f"  prompts: max abs err {stats['err']:.3e}", flush=True)
    slots = list(range(batch))
    for step in range(2):
        lg, nx = g.decode_step(slots, t)
        nx = [int(v) for v in nx.tolist()]
        for b in watched:
            lo, nb = o.step_token(watched[b], t[b], fl)
            _check_step(lg[b], lo, f"step {step} slot {b}", stats)
            nx[b] = nb
        t = nx
    print(f"  max abs err {stats['err']:.3e}, min margin {stats['margin']:.3e}, ties {stats['ties']}", flush=True)
    assert not stats["ties"], stats["ties"]


GOLDEN_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


@pytest.mark.parametrize("workload,name,batch,ctx,variant,mode", [
    ("cfg3", "qwen3-4b", 8, 2048, "mirrored", 0), ("cfg3", "qwen3-4b", 8, 2048, "plain", 2),
    ("cfg3", "qwen3-4b", 8, 2048, "plain", 0), ("cfg4", "qwen3-8b", 16, 4096, "mirrored", 0)])
def test_full_depth_full_context_against_offline_oracle(nnc, workload, name, batch, ctx, variant, mode):
    """Configs 3 and 4 at full depth AND full context: slot 0's prompt pass and 8 decode steps,
    teacher-forced on the oracle's tokens, against what the oracle wrote offline
    (tests/golden/make_full_depth_goldens.py; hours of CPU).  Decode runs alone (resident kernel)
    and as one column of a full batch (per-stage kernels).
      mirrored, mode 0  the default prompt pass (single-piece blocks + fp32-grade tail) against the
                        oracle that rounds where those blocks do: the stated bar, 3e-2.
      plain, mode 2     NNC_OPT_PREFILL_EXACT = 2 (two pieces at every length) against the exact
                        definition with only the 16-bit cache: the stated bar, 3e-2.
      plain, mode 0     the default prompt pass against the exact definition: how far single-piece
                        prompt blocks are from it at full depth.  Reported; bounded at 1e-1 (the
                        cache rows of 2032 positions x 36 layers carry bf16-grade noise on top of
                        their bf16 storage rounding: measured 6e-2, 1 % of the logit range); the
                        greedy tokens must still agree."""
    bar = 1e-1 if (variant == "plain" and mode == 0) else 3e-2
    print(f"case: {workload} full depth, full context, {variant} oracle values", flush=True)
    path = os.path.join(GOLDEN_DIR, f"{workload}_slot0_{variant}.npz")
    assert os.path.exists(path), f"{path} missing: run tests/golden/make_full_depth_goldens.py {workload}"
    z = np.load(path)
    with open(os.path.join(os.path.dirname(GOLDEN_DIR), "..", "oracle", "oracle.cpp"), "rb") as f:
        assert str(z["oracle_sha256"]) == hashlib.sha256(f.read()).hexdigest(), \
            "oracle.cpp changed since the expected values were written: regenerate them"
    assert int(z["context"]) == ctx and int(z["weight_seed"]) == synth.WEIGHT_SEED \
        and int(z["input_seed"]) == synth.INPUT_SEED and str(z["shape"]) == name
    want, nxt = z["logits"].astype(np.float64), z["next"]
    steps = len(nxt) - 1
    shape, _, g = _big_model(nnc, name, batch, ctx)
    g.set_option(nnc.OPT_PREFILL_EXACT, mode)
    toks = synth.tokens(ctx, shape.vocab, stream=int(z["stream"]))
    stats = dict(err=0.0, margin=np.inf, ties=[], bar=bar)
    lg, _ = g.prefill(0, toks)
    _check_step(lg, want[0], "prompt", stats)
    print(f"  prompt: max abs err {stats['err']:.3e}, margin {stats['margin']:.3e}", flush=True)
    for i in range(steps):                             # alone
        lg, _ = g.decode_step([0], [int(nxt[i])])
        _check_step(lg[0], want[i + 1], f"alone step {i}", stats)
    print(f"  alone: max abs err {stats['err']:.3e}", flush=True)
    g.kv_reset(-1)                                     # as column 0 of a full batch
    g.prefill(0, toks, want_logits=False)
    t = [int(nxt[0])]
    for b in range(1, batch):
        _, nx = g.prefill(b, synth.tokens(16 + 9 * b, shape.vocab, stream=50 + b))
        t.append(int(nx.item()))
    slots = list(range(batch))
    for i in range(steps):
        lg, nx = g.decode_step(slots, t)
        _check_step(lg[0], want[i + 1], f"batched step {i}", stats)
        t = [int(nxt[i + 1])] + [int(v) for v in nx.tolist()[1:]]
    g.set_option(nnc.OPT_PREFILL_EXACT, 0)
    print(f"  max abs err {stats['err']:.3e}, min margin {stats['margin']:.3e}, ties {stats['ties']}", flush=True)
    assert not stats["ties"], stats["ties"]
