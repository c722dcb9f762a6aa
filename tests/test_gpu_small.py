"""GPU parity on small shapes: every kernel family, ragged sizes, edge cases.

All calls go through the C ABI (ctypes binding).  Tolerances:
  fp32 models  : per-row infinity-norm relative error <= 1e-4 (the stated bar)
  bf16 models  : max abs logit error <= 3e-2 (the stated bar); these small models are
                 also held to 4e-3: fp32 accumulation plus an occasional one-ulp bf16
                 difference in a cached K/V element gives ~1e-3 here.
"""
import numpy as np
import pytest

import oracle
import synth
from parity_util import (SMALL_BF16, SMALL_F32, SMALL_G4, SMALL_LAYER_F32, oracle_flags,
                         oracle_prefill_like_library, prefill_blocks, rel_inf)

pytestmark = pytest.mark.gpu

BF16_ABS = 3e-2
BF16_ABS_TIGHT = 4e-3
# Prompt blocks of more than 512 tokens run with matrix-core inputs rounded to bf16 once; the
# oracle mirrors those rounding points block by block (parity_util.prefill_blocks), but the two
# sides round values that differ by fp32-vs-fp64 noise, some elements then round the other way
# (one ulp = 0.4 %) and the difference cascades.  The last 16 tokens of such a prompt take the
# fp32-grade path, and every shorter prompt carries two bf16 pieces per activation.
BF16_ABS_PROMPT = 2.5e-2
F32_REL = 1e-4


@pytest.fixture(scope="module")
def nnc():
    from paper_2512_21571_amd import binding
    binding.lib()
    return binding


def _pair(nnc, shape, max_batch, max_seq, weight_std=0.05, jitter=0.1, exact_prefill=True):
    """GPU model + oracle over the same blob.  exact_prefill selects the prompt path: fp32-grade
    activations in 21-token chunks (True) or the large-block matrix-core GEMMs (False)."""
    blob = synth.make_blob(shape, weight_std=weight_std, gain_jitter=jitter)
    g = nnc.Model(shape, blob, max_batch, max_seq)
    if shape.dtype != synth.F32 and shape.has_embed_and_head:
        g.set_option(nnc.OPT_PREFILL_EXACT, int(exact_prefill))
    return g, oracle.from_shape(shape, blob, max_batch, max_seq)


def _check_logits(shape, got, want, tight=BF16_ABS_TIGHT):
    got = got.double().cpu().numpy()
    assert np.isfinite(got).all()
    if shape.dtype == synth.F32:
        assert rel_inf(got, want) <= F32_REL
    else:
        err = np.abs(got - want).max()
        assert err <= BF16_ABS
        assert err <= tight, err


@pytest.mark.parametrize("exact", [True, False], ids=["exact-prompt", "bf16-prompt"])
@pytest.mark.parametrize("shape", [SMALL_BF16, SMALL_G4, SMALL_F32], ids=lambda s: s.name)
def test_prefill_then_decode_matches_oracle(nnc, shape, exact):
    print(f"case: prefill+decode {shape.name} exact={exact}", flush=True)
    if shape.dtype == synth.F32 and not exact:
        pytest.skip("fp32 models have one prompt path")
    g, o = _pair(nnc, shape, 2, 160, exact_prefill=exact)
    fl = oracle_flags(shape)
    toks = synth.tokens(70, shape.vocab)          # 70 = full 21/64-column chunks + a ragged tail
    tight = BF16_ABS_TIGHT
    lg, ng = g.prefill(0, toks)
    lo, no = o.prefill(0, toks, fl)
    _check_logits(shape, lg, lo, tight)
    assert int(ng.item()) == no
    t = no
    for step in range(70):                        # crosses the 64- and 128-position chunk edges
        lg, ng = g.decode_step([0], [t])
        lo, no = o.step_token(0, t, fl)
        _check_logits(shape, lg[0], lo, tight)
        assert int(ng.item()) == no, step
        t = no
    assert g.slot_len(0) == 140 and o.slot_len(0) == 140


@pytest.mark.parametrize("n", [1, 20, 21, 22, 42, 65])
def test_prefill_lengths_and_kv_rows(nnc, n):
    print(f"case: prefill length {n}", flush=True)
    shape = SMALL_BF16
    g, o = _pair(nnc, shape, 1, 80)
    fl = oracle_flags(shape)
    toks = synth.tokens(n, shape.vocab, stream=n)
    lg, _ = g.prefill(0, toks)
    lo, _ = o.prefill(0, toks, fl)
    _check_logits(shape, lg, lo)
    for layer in range(shape.n_layers):
        for which in (0, 1):
            got = g.kv_read(layer, 0, which, 0, n).double().cpu().numpy()
            want = o.kv_rows(layer, 0, which)
            # both sides store bf16; where the fp32 and fp64 pre-rounding values straddle a
            # rounding boundary they differ by one bf16 ulp, plus the pre-rounding difference
            # itself (visible only on elements near zero, whose ulp is tiny)
            ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-30))) - 7)
            # layer 0 sees only fp32-vs-fp64 noise before rounding; deeper layers also see
            # the effect of upstream one-ulp cache differences on their inputs
            pre = 1e-5 if layer == 0 else 3e-3
            excess = np.abs(got - want) - (ulp * 1.001 + pre)
            w = np.unravel_index(np.argmax(excess), excess.shape)
            assert excess[w] <= 0, (layer, which, w, got[w], want[w])
            # one differing element upstream perturbs every later activation by ~1e-4
            # relative, which in turn moves a few percent of the next layer's elements
            # across a rounding boundary; the first layer has no upstream
            assert np.mean(got != want) < (0.01 if layer == 0 else 0.15)


@pytest.mark.parametrize("n", [1, 15, 16, 17, 63, 64, 65, 127, 128, 129, 150, 256, 257, 300, 512, 513, 528, 529, 600, 900])
def test_large_block_prefill_lengths(nnc, n):
    print(f"case: large-block prefill length {n}", flush=True)
    shape = SMALL_G4
    g, o = _pair(nnc, shape, 1, 1024, exact_prefill=False)
    toks = synth.tokens(n, shape.vocab, stream=100 + n)
    one_piece = any(pc == 1 for _, _, pc in prefill_blocks(n))   # n > 528: a single-piece block, then the tail
    tight = BF16_ABS_PROMPT if one_piece else BF16_ABS_TIGHT
    lg, ng = g.prefill(0, toks)
    lo, no = oracle_prefill_like_library(o, 0, toks, shape)
    _check_logits(shape, lg, lo, tight)
    assert int(ng.item()) == no
    # the cache must be what the oracle's prompt pass cached: same rows in the same places.
    # Element-wise the two differ by an occasional bf16 ulp plus the noise of the inputs
    # upstream; a misplaced row, head or position would be off by O(1) everywhere.
    got = g.kv_read(shape.n_layers - 1, 0, 0, 0, n).double().cpu().numpy()
    want = o.kv_rows(shape.n_layers - 1, 0, 0)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-30))) - 7)
    if one_piece:
        assert np.all(np.abs(got - want) <= 2 * ulp + 3e-2)
        assert np.median(np.abs(got - want)) <= 4e-3
    else:
        assert np.all(np.abs(got - want) <= 1.001 * ulp + 3e-3)
        assert np.mean(got != want) < 0.15
    assert np.abs(want).mean() > 0.3
    # decode continues from that cache with exact activations
    t = no
    for _ in range(3):
        lg, ng = g.decode_step([0], [t])
        lo, t = o.step_token(0, t, oracle_flags(shape))
        _check_logits(shape, lg[0], lo, tight)
        assert int(ng.item()) == t


@pytest.mark.parametrize("tile", [0, 1, 2, 3, 4, 5, 6])
@pytest.mark.parametrize("n", [47, 300, 700])
def test_large_block_prefill_every_block_tile(nnc, n, tile):
    """Each GEMM block tile (64 x 128, 256 x 128, 128 x 128, 64 x 64, 192 x 128, 256 x 256, 192 x 256) forced on ragged
    small shapes.  The k order of every output element is the same in all of them, so the logits
    are bit-identical to those of the 256 x 128 tile -- except where a 64-row tile splits the k
    range of the narrow projections of a short block over several workgroups (partial sums added
    in a fixed order).  All match the oracle."""
    print(f"case: large-block prefill length {n}, forced block tile {tile}", flush=True)
    shape = SMALL_G4
    g, o = _pair(nnc, shape, 1, 800, exact_prefill=False)
    toks = synth.tokens(n, shape.vocab, stream=300 + n)
    one_piece = any(pc == 1 for _, _, pc in prefill_blocks(n))
    g.set_option(nnc.OPT_PREFILL_TILE, 1)
    ref, _ = g.prefill(0, toks)
    g.kv_reset(0)
    g.set_option(nnc.OPT_PREFILL_TILE, tile)
    lg, ng = g.prefill(0, toks)
    if tile in (1, 2, 4, 5, 6) or n > 512:
        assert np.array_equal(lg.cpu().numpy(), ref.cpu().numpy())
    else:
        # a partial-sum order that differs in the last bit can round a cached bf16 K / V element
        # the other way, which moves the logits by ~1e-4
        assert np.abs(lg.cpu().numpy() - ref.cpu().numpy()).max() <= 5e-4
    lo, no = oracle_prefill_like_library(o, 0, toks, shape)
    _check_logits(shape, lg, lo, BF16_ABS_PROMPT if one_piece else BF16_ABS_TIGHT)
    assert int(ng.item()) == no
    g.set_option(nnc.OPT_PREFILL_TILE, -1)
    g.kv_reset(0)
    la, na = g.prefill(0, toks)                      # the automatic choice
    _check_logits(shape, la, lo, BF16_ABS_PROMPT if one_piece else BF16_ABS_TIGHT)
    assert int(na.item()) == no


@pytest.mark.parametrize("ks", [2, 3, 4])
@pytest.mark.parametrize("tile", [0, 2, 3, 4, 5, 6])
def test_large_block_prefill_k_slices_on_every_block_tile(nnc, tile, ks):
    """The k range of the output and down projections split over `ks` workgroups per output tile
    (what the tile model picks for blocks whose tiles alone would leave most CUs idle): slice 0
    adds the residual, the others store partial sums that the next norm kernel adds in slice order.
    Every tile's kernel cuts the same k ranges and keeps the k order inside them, so for one slice
    count all tiles give the bits of the 256 x 128 tile; against the unsliced launch only the
    partial-sum order differs.  All match the oracle."""
    print(f"case: large-block prefill, forced block tile {tile}, {ks} k slices", flush=True)
    shape, n = SMALL_G4, 700
    g, o = _pair(nnc, shape, 1, 800, exact_prefill=False)
    toks = synth.tokens(n, shape.vocab, stream=1000 + n)
    g.set_option(nnc.OPT_PREFILL_TILE, 1)
    whole, _ = g.prefill(0, toks)
    g.kv_reset(0)
    g.set_option(nnc.OPT_PREFILL_KSLICES, ks)
    ref, _ = g.prefill(0, toks)
    g.kv_reset(0)
    g.set_option(nnc.OPT_PREFILL_TILE, tile)
    lg, ng = g.prefill(0, toks)
    assert np.array_equal(lg.cpu().numpy(), ref.cpu().numpy())
    # (a partial-sum order that differs in the last bit can round a cached bf16 K / V element the
    # other way, which moves the logits by ~1e-4)
    d = float(np.abs(lg.cpu().numpy() - whole.cpu().numpy()).max())
    assert 0.0 < d <= 5e-4, d                       # the slices were really taken, and change nothing else
    lo, no = oracle_prefill_like_library(o, 0, toks, shape)
    _check_logits(shape, lg, lo, BF16_ABS_PROMPT)
    assert int(ng.item()) == no
    lg2, n2 = g.decode_step([0], [no])              # the cache the sliced block left behind
    lo2, no2 = o.step_token(0, no, oracle_flags(shape))
    _check_logits(shape, lg2[0], lo2, BF16_ABS_PROMPT)
    assert int(n2.item()) == no2


@pytest.mark.parametrize("tile", [-1, 0, 1, 2, 3, 4, 5, 6])
def test_large_block_prefill_short_k_loops(nnc, tile):
    """A model so narrow that the GEMM k loops have 2 (QKV, gate|up) and 3 (down) steps:
    shorter than the register ring and than the three LDS stages of the block-tile kernels."""
    print(f"case: large-block prefill, hidden 64 / ffn 96, forced block tile {tile}", flush=True)
    shape = synth.ModelShape("narrow", hidden=64, n_layers=2, n_q_heads=2, n_kv_heads=1, head_dim=128,
                             ffn=96, vocab=512, dtype=synth.BF16)
    g, o = _pair(nnc, shape, 1, 256, exact_prefill=False)
    g.set_option(nnc.OPT_PREFILL_TILE, tile)
    toks = synth.tokens(200, shape.vocab, stream=9)
    lg, ng = g.prefill(0, toks)
    lo, no = oracle_prefill_like_library(o, 0, toks, shape)
    _check_logits(shape, lg, lo, BF16_ABS_TIGHT)
    assert int(ng.item()) == no


@pytest.mark.parametrize("attn", [0, 1, 2, 3])
@pytest.mark.parametrize("n", [40, 330, 700])
def test_large_block_prefill_every_attention_shape(nnc, n, attn):
    """Prompt attention launch shapes (one or two 64-token blocks per workgroup, one or two
    heads per wave) forced on prompts with an odd and an even number of blocks: a wave's
    arithmetic per head is the same in all of them, so the logits are bit-identical to the
    automatic choice, and they match the oracle."""
    print(f"case: large-block prefill length {n}, forced attention shape {attn}", flush=True)
    shape = SMALL_G4
    g, o = _pair(nnc, shape, 1, 800, exact_prefill=False)
    toks = synth.tokens(n, shape.vocab, stream=500 + n)
    one_piece = any(pc == 1 for _, _, pc in prefill_blocks(n))
    ref, _ = g.prefill(0, toks)
    g.kv_reset(0)
    g.set_option(nnc.OPT_PREFILL_ATTN, attn)
    lg, ng = g.prefill(0, toks)
    assert np.array_equal(lg.cpu().numpy(), ref.cpu().numpy())
    lo, no = oracle_prefill_like_library(o, 0, toks, shape)
    _check_logits(shape, lg, lo, BF16_ABS_PROMPT if one_piece else BF16_ABS_TIGHT)
    assert int(ng.item()) == no


@pytest.mark.parametrize("planner", [0, 1], ids=["hand-rules", "planner"])
@pytest.mark.parametrize("batch", [1, 3, 16])
def test_fused_qk_norm_rope_append_equals_separate_kernel(nnc, batch, planner):
    """Per-stage decode passes with QK-norm / RoPE / cache append inside the attention kernel and
    in a kernel of their own: the same arithmetic in the same order, so the same bits -- over
    steps that cross a 64-position chunk boundary, ragged contexts, eager and captured.  With the
    analytic planner the fused kernel may receive the QKV projection as k-slice partial sums and
    add them itself (another summation order): then the two agree to fp32 rounding."""
    print(f"case: fused vs separate QK-norm/RoPE/append, B={batch}, planner={planner}", flush=True)
    shape = SMALL_G4
    runs = []
    for fused in (0, 1):
        g, _ = _pair(nnc, shape, batch, 260)
        g.set_option(nnc.OPT_PERSISTENT, 0)
        g.set_option(nnc.OPT_PLANNER, planner)
        g.set_option(nnc.OPT_FUSE_QK, fused)
        firsts = []
        for s in range(batch):
            _, nx = g.prefill(s, synth.tokens(55 + 9 * s, shape.vocab, stream=40 + s))
            firsts.append(int(nx.item()))
        slots = list(range(batch))
        toks, logits = g.decode_greedy(slots, firsts, 14, want_logits=True)
        lg, ng = g.decode_step(slots, toks[-1].cpu().numpy().tolist())
        k = g.kv_read(1, 0, 0, 0, 55 + 15)
        v = g.kv_read(1, 0, 1, 0, 55 + 15)
        runs.append((toks.cpu().numpy().copy(), logits.cpu().numpy().copy(), lg.cpu().numpy().copy(),
                     k.cpu().numpy().copy(), v.cpu().numpy().copy()))
    if not planner:
        for a, b in zip(runs[0], runs[1]):
            assert np.array_equal(a, b)
        return
    (t0, l0, s0, k0, v0), (t1, l1, s1, k1, v1) = runs
    assert np.array_equal(t0, t1)
    assert np.abs(l0 - l1).max() <= 2e-4 and np.abs(s0 - s1).max() <= 2e-4
    for a, b in ((k0, k1), (v0, v1)):      # cache rows: the same 16-bit value, or its neighbour where the sums straddle a tie
        assert np.all(np.abs(a - b) <= np.abs(a) * 2.0 ** -7 + 1e-30) and np.mean(a != b) < 0.02


@pytest.mark.parametrize("shape,fuse", [(SMALL_BF16, 1), (SMALL_G4, 0)], ids=["small-bf16-fused", "small-g4-separate"])
def test_batched_decode_mixed_lengths_up_to_4k(nnc, shape, fuse):
    """Three slots of one batch at very different lengths (100, 2040 and 4090 cached positions,
    i.e. 2 to 65 chunks of the decode attention, the two long ones crossing 2048 and 4096 while
    decoding); logits and greedy tokens are checked against the oracle at every step, prompt
    included (fp32-grade prompt path, which runs the same attention kernel)."""
    print(f"case: long-context batched decode {shape.name} fuse={fuse}", flush=True)
    lens = [2040, 4090, 100]
    g, o = _pair(nnc, shape, 3, 4120, exact_prefill=True)
    g.set_option(nnc.OPT_FUSE_QK, fuse)
    fl = oracle_flags(shape)
    cur = []
    for b, n in enumerate(lens):
        toks = synth.tokens(n, shape.vocab, stream=40 + b)
        lg, ng = g.prefill(b, toks)
        lo, no = o.prefill(b, toks, fl)
        _check_logits(shape, lg, lo)
        assert int(ng.item()) == no
        cur.append(no)
    for step in range(14):                         # slot 0 crosses 2048, slot 1 crosses 4096
        lg, ng = g.decode_step([0, 1, 2], cur)
        for b in range(3):
            lo, no = o.step_token(b, cur[b], fl)
            _check_logits(shape, lg[b], lo)
            assert int(ng[b].item()) == no, (step, b)
            cur[b] = no
    assert g.slot_len(1) == 4104


def test_prompt_tail_beside_the_last_block_equals_tail_after_it(nnc):
    """The fp32-grade pass over a long prompt's last tokens runs on the library's second stream
    beside the last block (default) or after it on the model's stream: same bits, for one block,
    two blocks, prompts back to back in one model, and the decode steps that follow."""
    shape = SMALL_G4
    blob = synth.make_blob(shape, weight_std=0.05, gain_jitter=0.1)
    out = {}
    for overlap in (1, 0):
        print(f"case: prompt tail overlap={overlap}", flush=True)
        g = nnc.Model(shape, blob, 3, 2300)
        g.set_option(nnc.OPT_PREFILL_EXACT, 0)
        g.set_option(nnc.OPT_TAIL_OVERLAP, overlap)
        res = []
        firsts = []
        for b, n in enumerate([700, 2200, 1300]):
            lg, nx = g.prefill(b, synth.tokens(n, shape.vocab, stream=70 + b))
            res.append(lg.cpu().numpy().copy())
            firsts.append(int(nx.item()))
        toks, logits = g.decode_greedy([0, 1, 2], firsts, 3, want_logits=True)
        res.append(logits.cpu().numpy().copy())
        res.append(toks.cpu().numpy().copy())
        out[overlap] = (res, firsts)
        del g
    assert out[1][1] == out[0][1]
    for a, b in zip(out[1][0], out[0][0]):
        assert np.array_equal(a, b)
    # and the default path against the oracle
    o = oracle.from_shape(shape, blob, 1, 800)
    lo, no = oracle_prefill_like_library(o, 0, synth.tokens(700, shape.vocab, stream=70), shape)
    assert np.abs(out[1][0][0].astype(np.float64) - lo).max() <= BF16_ABS_PROMPT
    assert out[1][1][0] == no


def test_random_requests_against_oracle(nnc):
    """Seeded random requests (shape, batch, ragged prompt lengths across the block and piece
    boundaries, decode steps, forced kernel shapes, fused / separate kernels, resident / per-stage
    decode) against the oracle: logits within tolerance at every step, every greedy token equal
    unless the oracle's top-2 margin is within 4x that step's measured error (a tie within error:
    counted and printed).  A sequence whose on-device greedy loop leaves the oracle's tokens at
    such a tie is decoded again, teacher-forced on the oracle's tokens, so that every step of
    every request is compared."""
    import random
    rng = random.Random(20251)
    ties = []
    for case in range(14):
        shape = rng.choice([SMALL_BF16, SMALL_G4])
        batch = rng.choice([1, 1, 2, 3, 5])
        n = rng.choice([rng.randint(1, 70), rng.randint(60, 520), rng.randint(513, 900)])
        steps = rng.randint(1, 6)
        tile, attn = rng.choice([-1, -1, 0, 1, 2, 3, 4]), rng.choice([-1, -1, 0, 1, 2, 3])
        fuse, pers = rng.choice([0, 1]), rng.choice([0, 1])
        print(f"case: random request {case}: {shape.name} B={batch} n={n} steps={steps} tile={tile} "
              f"attn={attn} fuse={fuse} resident={pers}", flush=True)
        g, o = _pair(nnc, shape, batch, n + steps + 8, exact_prefill=False)
        g.set_option(nnc.OPT_PREFILL_TILE, tile)
        g.set_option(nnc.OPT_PREFILL_ATTN, attn)
        g.set_option(nnc.OPT_FUSE_QK, fuse)
        g.set_option(nnc.OPT_PERSISTENT, pers)
        fl = oracle_flags(shape)
        firsts, prompts = [], []
        for b in range(batch):
            nb = max(1, n - 7 * b)
            toks = synth.tokens(nb, shape.vocab, stream=1000 * case + b)
            prompts.append(toks)
            lg, ng = g.prefill(b, toks)
            lo, no = oracle_prefill_like_library(o, b, toks, shape)
            one_piece = any(pc == 1 for _, _, pc in prefill_blocks(nb))
            _check_logits(shape, lg, lo, BF16_ABS_PROMPT if one_piece else BF16_ABS_TIGHT)
            assert int(ng.item()) == no
            firsts.append(no)
        toks_g, logits_g = g.decode_greedy(list(range(batch)), firsts, steps, want_logits=True)
        cur = list(firsts)
        left = [False] * batch            # the device loop of this sequence has left the oracle's tokens
        fed, want = [], []                # per step: the oracle's input tokens, its logits
        for s_ in range(steps):
            fed.append(list(cur))
            want.append([])
            for b in range(batch):
                lo, nx = o.step_token(b, cur[b], fl)
                want[-1].append(lo)
                if not left[b]:
                    _check_logits(shape, logits_g[s_, b], lo, BF16_ABS_PROMPT)
                    if int(toks_g[s_, b].item()) != nx:
                        err = np.abs(logits_g[s_, b].double().cpu().numpy() - lo).max()
                        top = np.sort(lo)[-2:]
                        assert top[1] - top[0] < 4 * err, (case, s_, b, top[1] - top[0], err)
                        ties.append((case, s_, b, float(top[1] - top[0]), float(err)))
                        left[b] = True
                cur[b] = nx
        if any(left):
            g.kv_reset(-1)
            for b in range(batch):
                g.prefill(b, prompts[b], want_logits=False)
            for s_ in range(steps):
                lg, _ = g.decode_step(list(range(batch)), fed[s_])
                for b in range(batch):
                    _check_logits(shape, lg[b], want[s_][b], BF16_ABS_PROMPT)
    print(f"ties within error (case, step, slot, oracle margin, max abs error): {ties}", flush=True)
    assert len(ties) <= 1, ties


@pytest.mark.parametrize("shape", [SMALL_BF16, SMALL_G4], ids=lambda s: s.name)
def test_default_long_prompt_against_the_unmirrored_oracle(nnc, shape):
    """A 2100-token prompt in the default mode (a 2084-token block with matrix-core inputs
    rounded to bf16 once, then the fp32-grade 16-token tail) against the oracle with NO mirrored rounding, only the 16-bit cache: the stated bar
    (3e-2, greedy agreement) must hold against the exact definition too, and the decode steps
    that follow read that cache."""
    print(f"case: default-mode 2100-token prompt vs the plain oracle, {shape.name}", flush=True)
    g, o = _pair(nnc, shape, 1, 2120, exact_prefill=False)
    toks = synth.tokens(2100, shape.vocab, stream=33)
    fl = oracle_flags(shape)
    lg, ng = g.prefill(0, toks)
    lo, no = o.prefill(0, toks, fl)
    errs = [float(np.abs(lg.double().cpu().numpy() - lo).max())]
    assert int(ng.item()) == no or np.sort(lo)[-1] - np.sort(lo)[-2] < 4 * errs[0]
    t = no
    for _ in range(6):
        lg, ng = g.decode_step([0], [t])
        lo, no = o.step_token(0, t, fl)
        errs.append(float(np.abs(lg[0].double().cpu().numpy() - lo).max()))
        assert int(ng.item()) == no or np.sort(lo)[-1] - np.sort(lo)[-2] < 4 * errs[-1]
        t = no
    print(f"  max abs logit error vs the plain oracle: prompt {errs[0]:.3e}, decode {max(errs[1:]):.3e}; "
          f"|logit| max {np.abs(lo).max():.2f}", flush=True)
    assert max(errs) <= BF16_ABS


def test_large_block_prefill_two_pieces_at_any_length(nnc):
    print("case: large-block prefill, 600 tokens, two pieces forced", flush=True)
    shape = SMALL_G4
    g, o = _pair(nnc, shape, 1, 640, exact_prefill=False)
    g.set_option(nnc.OPT_PREFILL_EXACT, 2)
    toks = synth.tokens(600, shape.vocab, stream=41)
    lg, ng = g.prefill(0, toks)
    lo, no = o.prefill(0, toks, oracle_flags(shape))
    _check_logits(shape, lg, lo, BF16_ABS_TIGHT)
    assert int(ng.item()) == no


def test_batched_decode_long_contexts(nnc):
    """16 sequences with 2100-position contexts: many chunks per sequence in the batched
    attention kernels, ragged last chunks."""
    print("case: batched decode, 16 x 2100 positions", flush=True)
    shape = SMALL_BF16
    B = 16
    g, o = _pair(nnc, shape, B, 2120, exact_prefill=False)
    t = []
    for b in range(B):
        toks = synth.tokens(2100 - 3 * b, shape.vocab, stream=500 + b)
        g.prefill(b, toks, want_logits=False)
        _, nxt = oracle_prefill_like_library(o, b, toks, shape)
        t.append(nxt)
    for step in range(2):
        lg, ng = g.decode_step(list(range(B)), t)
        nxt = []
        for b in range(B):
            lo, nb = o.step_token(b, t[b], oracle_flags(shape))
            _check_logits(shape, lg[b], lo, BF16_ABS_PROMPT)
            assert int(ng[b].item()) == nb, (step, b)
            nxt.append(nb)
        t = nxt


def test_multi_block_prefill_long_context(nnc):
    print("case: prompt of several blocks (2048 + 736 single-piece, 16 fp32-grade)", flush=True)
    shape = SMALL_BF16
    g, o = _pair(nnc, shape, 1, 2900, exact_prefill=False)
    g.set_option(nnc.OPT_PREFILL_BLOCK, 2048)
    toks = synth.tokens(2800, shape.vocab, stream=77)
    assert [(nb, pc) for _, nb, pc in prefill_blocks(2800, 2048)] == [(2048, 1), (736, 1), (16, 3)]
    lg, ng = g.prefill(0, toks)
    lo, no = oracle_prefill_like_library(o, 0, toks, shape, 2048)
    _check_logits(shape, lg, lo, BF16_ABS_PROMPT)
    assert int(ng.item()) == no
    for attn in (1, 3):                                     # paired attention blocks on a block that starts mid-context
        g.kv_reset(0)
        g.set_option(nnc.OPT_PREFILL_ATTN, attn)
        l2, _ = g.prefill(0, toks)
        assert np.array_equal(l2.cpu().numpy(), lg.cpu().numpy())
    g.set_option(nnc.OPT_PREFILL_ATTN, -1)
    lg, ng = g.decode_step([0], [no])                       # 44 attention chunks in the resident kernel
    lo, n2 = o.step_token(0, no, oracle_flags(shape))
    _check_logits(shape, lg[0], lo, BF16_ABS_PROMPT)
    assert int(ng.item()) == n2


def test_default_blocks_of_4096_tokens(nnc):
    print("case: prompt of 4300 tokens in default blocks (4096 single-piece + 188 two-piece, 16 fp32-grade)", flush=True)
    shape = SMALL_G4
    g, o = _pair(nnc, shape, 1, 4320, exact_prefill=False)
    toks = synth.tokens(4300, shape.vocab, stream=78)
    assert [(nb, pc) for _, nb, pc in prefill_blocks(4300)] == [(4096, 1), (188, 2), (16, 3)]
    lg, ng = g.prefill(0, toks)
    lo, no = oracle_prefill_like_library(o, 0, toks, shape)
    _check_logits(shape, lg, lo, BF16_ABS_PROMPT)
    assert int(ng.item()) == no
    # the blocking changes no rounding point of blocks beyond 512 tokens: 2048-token blocks give
    # logits within the same distance of the same oracle values
    g.kv_reset(0)
    g.set_option(nnc.OPT_PREFILL_BLOCK, 2048)
    l2, n2 = g.prefill(0, toks)
    _check_logits(shape, l2, lo, BF16_ABS_PROMPT)
    assert int(n2.item()) == no


@pytest.mark.parametrize("batch", [2, 5, 8, 16])
def test_batched_decode_equals_independent_sequences(nnc, batch):
    print(f"case: batched decode B={batch}", flush=True)
    shape = SMALL_G4
    g, o = _pair(nnc, shape, batch, 120)
    fl = oracle_flags(shape)
    lens = [3 + 7 * i for i in range(batch)]                       # ragged contexts, some past 64
    nxt = []
    for s in range(batch):
        toks = synth.tokens(lens[s], shape.vocab, stream=s)
        g.prefill(s, toks, want_logits=False)
        _, n_o = o.prefill(s, toks, fl)
        nxt.append(n_o)
    slots = list(range(batch))[::-1]                               # slot order != column order
    for step in range(3):
        lg, ng = g.decode_step(slots, [nxt[s] for s in slots])
        ng = ng.cpu().numpy()
        for col, s in enumerate(slots):
            lo, n_o = o.step_token(s, nxt[s], fl)
            _check_logits(shape, lg[col], lo)
            assert int(ng[col]) == n_o
            nxt[s] = n_o


@pytest.mark.parametrize("persistent", [1, 0], ids=["resident", "per-stage"])
@pytest.mark.parametrize("batch", [1, 3])
def test_decode_from_empty_slots(nnc, batch, persistent):
    """No prompt at all: the first decode step runs at position 0 on an empty cache (the attention
    kernels then read only rows that were never written, with weight zero: the cache is
    zero-filled at create so that these are finite), the following ones on what the steps appended."""
    print(f"case: decode from empty slots, B={batch}, persistent={persistent}", flush=True)
    shape = SMALL_G4
    g, o = _pair(nnc, shape, batch, 80)
    g.set_option(nnc.OPT_PERSISTENT, persistent)
    fl = oracle_flags(shape)
    t = [int(v) for v in synth.tokens(batch, shape.vocab, stream=9)]
    for step in range(70):                     # crosses the first 64-position chunk boundary
        lg, ng = g.decode_step(list(range(batch)), t)
        nxt = []
        for b in range(batch):
            lo, nb = o.step_token(b, t[b], fl)
            _check_logits(shape, lg[b], lo)
            assert int(ng[b].item()) == nb, (step, b)
            nxt.append(nb)
        t = nxt


def test_hidden_state_layer_fp32(nnc):
    print("case: hidden-state layer fp32", flush=True)
    shape = SMALL_LAYER_F32
    g, o = _pair(nnc, shape, 2, 40, weight_std=0.05)
    x = synth.activations(24, shape.hidden)
    y = g.prefill_hidden(0, x[:16]).double().cpu().numpy()
    for t in range(16):
        want = o.step_hidden(0, x[t].astype(np.float64))
        assert rel_inf(y[t], want) <= F32_REL
    for t in range(16, 24):
        yg = g.decode_step_hidden([0], x[t:t + 1]).double().cpu().numpy()[0]
        want = o.step_hidden(0, x[t].astype(np.float64))
        assert rel_inf(yg, want) <= F32_REL


def test_greedy_loop_graph_and_eager_agree_with_oracle(nnc):
    print("case: greedy loop graph/eager", flush=True)
    shape = SMALL_BF16
    g, o = _pair(nnc, shape, 1, 200)
    fl = oracle_flags(shape)
    toks = synth.tokens(20, shape.vocab)
    _, first = o.prefill(0, toks, fl)
    want = []
    t = first
    for _ in range(120):
        _, t = o.step_token(0, t, fl)
        want.append(t)
    outs = {}
    # (persistent kernel, graph replay) x on/off: resident kernel, per-stage kernels in a
    # captured graph, per-stage kernels launched eagerly
    for mode in ((1, 1), (0, 1), (0, 0)):
        g.kv_reset(0)
        g.set_option(nnc.OPT_PERSISTENT, mode[0])
        g.set_option(nnc.OPT_GRAPH, mode[1])
        g.prefill(0, toks, want_logits=False)
        got, _ = g.decode_greedy([0], [first], 120)
        outs[mode] = got.cpu().numpy()[:, 0]
        assert g.slot_len(0) == 140
        assert np.array_equal(outs[mode], np.array(want)), mode
    # replay through the captured graph a second time, with eager work in between
    g.kv_reset(0)
    g.set_option(nnc.OPT_GRAPH, 1)
    g.prefill(0, toks, want_logits=False)
    again, _ = g.decode_greedy([0], [first], 120)
    assert np.array_equal(again.cpu().numpy()[:, 0], outs[(0, 1)])
    # and the resident kernel again after the per-stage path has run
    g.kv_reset(0)
    g.set_option(nnc.OPT_PERSISTENT, 1)
    g.prefill(0, toks, want_logits=False)
    again, _ = g.decode_greedy([0], [first], 120)
    assert np.array_equal(again.cpu().numpy()[:, 0], outs[(1, 1)])


def test_reset_replay_and_error_paths(nnc):
    print("case: reset/replay/errors", flush=True)
    shape = SMALL_BF16
    g, _ = _pair(nnc, shape, 2, 8)
    toks = synth.tokens(6, shape.vocab)
    a, _ = g.prefill(0, toks)
    a = a.cpu().numpy()
    g.kv_reset(0)
    b, _ = g.prefill(0, toks)
    assert np.array_equal(a, b.cpu().numpy())
    with pytest.raises(nnc.NncError) as e:
        g.prefill(0, synth.tokens(3, shape.vocab))          # 6 + 3 > 8
    assert e.value.status == nnc.E_KV_FULL and g.slot_len(0) == 6
    with pytest.raises(nnc.NncError) as e:
        g.decode_step([0, 0], [1, 2])
    assert e.value.status == nnc.E_ARG
    with pytest.raises(nnc.NncError) as e:
        g.decode_step([2], [1])
    assert e.value.status == nnc.E_ARG
    with pytest.raises(nnc.NncError) as e:
        g.decode_step([1], [shape.vocab])
    assert e.value.status == nnc.E_ARG
    with pytest.raises(nnc.NncError) as e:
        g.prefill_hidden(0, np.zeros((1, shape.hidden), np.float32))
    assert e.value.status == nnc.E_STATE
    g.decode_step([0], [1])
    g.decode_step([0], [1])
    with pytest.raises(nnc.NncError) as e:
        g.decode_step([0], [1])
    assert e.value.status == nnc.E_KV_FULL


@pytest.mark.parametrize("shape", [SMALL_BF16, SMALL_G4, SMALL_F32], ids=lambda s: s.name)
@pytest.mark.parametrize("batch", [1, 3, 16])
def test_norm_in_the_gemm_tail_equals_the_norm_kernel(nnc, shape, batch):
    """Per-stage decode passes with the RMSNorm after the output / down projections run in the
    tail of those GEMM launches, and in a kernel of its own: the same arithmetic in the same
    order, so the same bits (logits, tokens, cache rows), eager and captured, over ragged contexts."""
    print(f"case: norm in the GEMM tail vs norm kernel, {shape.name}, B={batch}", flush=True)
    runs = []
    for fused in (0, 1):
        g, _ = _pair(nnc, shape, batch, 200)
        g.set_option(nnc.OPT_PERSISTENT, 0)
        g.set_option(nnc.OPT_FUSE_NORM, fused)
        firsts = []
        for s_ in range(batch):
            _, nx = g.prefill(s_, synth.tokens(40 + 7 * s_, shape.vocab, stream=70 + s_))
            firsts.append(int(nx.item()))
        slots = list(range(batch))
        toks, logits = g.decode_greedy(slots, firsts, 6, want_logits=True)   # eager passes (logits wanted)
        toks2, _ = g.decode_greedy(slots, toks[-1].cpu().numpy().tolist(), 6)  # captured graph
        lg, ng = g.decode_step(slots, toks2[-1].cpu().numpy().tolist())
        g.synchronize()
        k = g.kv_read(shape.n_layers - 1, 0, 0, 0, 40 + 13)
        runs.append((toks.cpu().numpy().copy(), logits.cpu().numpy().copy(), toks2.cpu().numpy().copy(),
                     lg.cpu().numpy().copy(), ng.cpu().numpy().copy(), k.cpu().numpy().copy()))
    for a, b in zip(runs[0], runs[1]):
        assert np.array_equal(a, b)


def test_norm_tail_gives_up_cleanly_and_reports_it(nnc):
    """Failure path of the norm tail, forced from the host: with a spin limit of one poll a
    workgroup that finds the others not finished yet gives up instead of waiting; the launch ends
    normally, and the library reports the failure on synchronize and refuses further decode calls."""
    print("case: norm tail give-up path (spin limit 1)", flush=True)
    shape = SMALL_BF16
    blob = synth.make_blob(shape, weight_std=0.05)
    g = nnc.Model(shape, blob, 16, 64)
    firsts = []
    for s_ in range(16):
        _, nx = g.prefill(s_, synth.tokens(9, shape.vocab, stream=s_))
        firsts.append(int(nx.item()))
    g.set_option(nnc.OPT_FUSE_NORM, 1)
    g.set_option(nnc.OPT_SPIN_LIMIT, 1)
    g.decode_greedy(list(range(16)), firsts, 8)
    with pytest.raises(nnc.NncError) as ei:
        g.synchronize()
    assert ei.value.status == nnc.E_DEVICE
    with pytest.raises(nnc.NncError):
        g.decode_step(list(range(16)), firsts)


def test_resident_kernel_gives_up_cleanly_and_reports_it(nnc):
    """Failure path of the resident decode kernel, forced from the host: with a spin limit of
    one poll every wait that is not satisfied at once gives up, all workgroups leave through
    the same exit (no hang, no fault), and the library reports the failure on synchronize and
    refuses further decode calls on that model.  A fresh model is unaffected."""
    print("case: resident kernel give-up path (spin limit 1)", flush=True)
    shape = SMALL_BF16
    blob = synth.make_blob(shape, weight_std=0.05)
    g = nnc.Model(shape, blob, 1, 64)
    toks = synth.tokens(9, shape.vocab)
    _, nxt = g.prefill(0, toks)
    first = int(nxt.item())
    g.set_option(nnc.OPT_SPIN_LIMIT, 1)
    g.decode_greedy([0], [first], 4)            # enqueued; the kernel gives up inside
    with pytest.raises(nnc.NncError) as ei:
        g.synchronize()
    assert ei.value.status == nnc.E_DEVICE
    with pytest.raises(nnc.NncError):
        g.decode_step([0], [first])
    g2 = nnc.Model(shape, blob, 1, 64)          # same weights, new model: works
    _, nxt2 = g2.prefill(0, toks)
    assert int(nxt2.item()) == first
    out, _ = g2.decode_greedy([0], [first], 4)
    g2.synchronize()
    assert out.shape[0] == 4
