"""GPU parity of the binary16 ("F16") variant: the paper's own 16-bit precision (Section 4,
experimental setup: Qwen3-0.6B in F32 / F16, Qwen3-1.7B in F16).

Weights and the KV cache are IEEE binary16, accumulation is fp32, activations enter the matrix
cores as binary16 pieces (same structure as the bf16 variant; same kernels, instantiated for the
other format).  The oracle widens the binary16 blob and rounds cache rows (and, for mirrored
prompt blocks, the matrix-core inputs) to binary16 (ORC_ROUND_F16).  Tolerance: the stated
16-bit bar, max abs logit error <= 3e-2 with greedy agreement; binary16 has three more
significant bits than bf16, and the small models are held to 2e-3.
"""
import numpy as np
import pytest

import oracle
import synth
from parity_util import (SMALL_F16, SMALL_G4_F16, oracle_flags, oracle_prefill_like_library, prefill_blocks,
                         top2_margin)

pytestmark = pytest.mark.gpu

F16_ABS, F16_ABS_TIGHT, F16_ABS_PROMPT = 3e-2, 2e-3, 1e-2


@pytest.fixture(scope="module")
def nnc():
    from paper_2512_21571_amd import binding
    binding.lib()
    return binding


def _pair(nnc, shape, max_batch, max_seq, exact_prefill):
    blob = synth.make_blob(shape, weight_std=0.05, gain_jitter=0.1)
    g = nnc.Model(shape, blob, max_batch, max_seq)
    g.set_option(nnc.OPT_PREFILL_EXACT, int(exact_prefill))
    return g, oracle.from_shape(shape, blob, max_batch, max_seq)


def _check(got, want, tight):
    got = got.double().cpu().numpy()
    assert np.isfinite(got).all()
    err = float(np.abs(got - want).max())
    assert err <= F16_ABS and err <= tight, err
    return err


@pytest.mark.parametrize("exact", [True, False], ids=["chunk-prompt", "block-prompt"])
@pytest.mark.parametrize("shape", [SMALL_F16, SMALL_G4_F16], ids=lambda s: s.name)
def test_f16_prefill_then_decode_matches_oracle(nnc, shape, exact):
    print(f"case: binary16 prefill+decode {shape.name} exact={exact}", flush=True)
    g, o = _pair(nnc, shape, 2, 160, exact)
    fl = oracle_flags(shape)
    assert fl & oracle.ROUND_F16
    toks = synth.tokens(70, shape.vocab)
    lg, ng = g.prefill(0, toks)
    lo, no = o.prefill(0, toks, fl)
    worst = _check(lg, lo, F16_ABS_TIGHT)
    assert int(ng.item()) == no
    t = no
    for step in range(70):                        # resident kernel; crosses the 64- and 128-position chunk edges
        lg, ng = g.decode_step([0], [t])
        lo, no = o.step_token(0, t, fl)
        worst = max(worst, _check(lg[0], lo, F16_ABS_TIGHT))
        assert int(ng.item()) == no, step
        t = no
    print(f"  max abs logit error {worst:.3e}", flush=True)
    # the cached rows are binary16 values of the oracle's rows (one ulp where the two sides round apart)
    for which in (0, 1):
        got = g.kv_read(1, 0, which, 0, 140).double().cpu().numpy()
        want = o.kv_rows(1, 0, which, 140)
        # one binary16 ulp where the two sides' pre-rounding values straddle a rounding boundary,
        # plus the pre-rounding difference itself (layer 1 sees the effect of upstream one-ulp
        # cache differences on its inputs)
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 2.0 ** -14))) - 10)
        assert np.all(np.abs(got - want) <= ulp * 1.001 + 5e-4)
        assert np.mean(got != want) < 0.15


@pytest.mark.parametrize("n", [300, 700, 2100])
def test_f16_large_block_prompts(nnc, n):
    """Two-piece blocks (<= 512 tokens), single-piece blocks mirrored by the oracle, the fp32-grade tail."""
    print(f"case: binary16 large-block prompt of {n} tokens", flush=True)
    shape = SMALL_G4_F16
    g, o = _pair(nnc, shape, 1, n + 16, False)
    toks = synth.tokens(n, shape.vocab, stream=n)
    one_piece = any(pc == 1 for _, _, pc in prefill_blocks(n))
    lg, ng = g.prefill(0, toks)
    lo, no = oracle_prefill_like_library(o, 0, toks, shape)
    err = _check(lg, lo, F16_ABS_PROMPT if one_piece else F16_ABS_TIGHT)
    print(f"  max abs logit error {err:.3e} (single-piece blocks: {one_piece})", flush=True)
    assert int(ng.item()) == no
    lg, ng = g.decode_step([0], [no])
    lo, n2 = o.step_token(0, no, oracle_flags(shape))
    _check(lg[0], lo, F16_ABS_PROMPT if one_piece else F16_ABS_TIGHT)
    assert int(ng.item()) == n2


@pytest.mark.parametrize("tile", [2, 4, 5, 6])
def test_f16_block_tile_256x256_equals_256x128(nnc, tile):
    """The other block tiles of the prompt GEMMs (128 / 192 x 128; 256 / 192 x 256 with the
    accumulators named in inline assembly and their own binary16 instruction string) give the bits
    of the 256 x 128 tile.  (They did not while the compiler was free to fold the SwiGLU product
    into the binary16 conversion for some elements of the unrolled epilogue and not for others.)"""
    print(f"case: binary16 large-block prompt, forced block tile {tile}", flush=True)
    shape = SMALL_G4_F16
    g, _ = _pair(nnc, shape, 1, 720, False)
    toks = synth.tokens(700, shape.vocab, stream=77)
    g.set_option(nnc.OPT_PREFILL_TILE, 1)
    ref, _ = g.prefill(0, toks)
    g.kv_reset(0)
    g.set_option(nnc.OPT_PREFILL_TILE, tile)
    lg, _ = g.prefill(0, toks)
    assert np.array_equal(lg.cpu().numpy(), ref.cpu().numpy())


@pytest.mark.parametrize("tile", [0, 2, 5, 6])
def test_f16_block_tiles_with_k_slices(nnc, tile):
    """The residual projections of a block in three k slices: every tile's kernel gives the bits of
    the 256 x 128 tile for the same slice count, close to the unsliced result."""
    print(f"case: binary16 large-block prompt, forced block tile {tile}, 3 k slices", flush=True)
    shape = SMALL_G4_F16
    g, _ = _pair(nnc, shape, 1, 720, False)
    toks = synth.tokens(700, shape.vocab, stream=78)
    g.set_option(nnc.OPT_PREFILL_TILE, 1)
    whole, _ = g.prefill(0, toks)
    g.kv_reset(0)
    g.set_option(nnc.OPT_PREFILL_KSLICES, 3)
    ref, _ = g.prefill(0, toks)
    g.kv_reset(0)
    g.set_option(nnc.OPT_PREFILL_TILE, tile)
    lg, _ = g.prefill(0, toks)
    assert np.array_equal(lg.cpu().numpy(), ref.cpu().numpy())
    d = float(np.abs(lg.cpu().numpy() - whole.cpu().numpy()).max())
    assert 0.0 < d <= 5e-4, d


@pytest.mark.parametrize("batch,fuse", [(5, 1), (16, 0)])
def test_f16_batched_decode(nnc, batch, fuse):
    print(f"case: binary16 batched decode, {batch} sequences, fused QK-norm {fuse}", flush=True)
    shape = SMALL_F16
    g, o = _pair(nnc, shape, batch, 400, False)
    g.set_option(nnc.OPT_FUSE_QK, fuse)
    fl = oracle_flags(shape)
    t = []
    for b in range(batch):
        toks = synth.tokens(30 + 23 * b, shape.vocab, stream=b)      # ragged contexts, up to 6 chunks
        g.prefill(b, toks, want_logits=False)
        _, nb = o.prefill(b, toks, fl)
        t.append(nb)
    for step in range(3):
        lg, ng = g.decode_step(list(range(batch)), t)
        nxt = []
        for b in range(batch):
            lo, nb = o.step_token(b, t[b], fl)
            _check(lg[b], lo, F16_ABS_TIGHT)
            assert int(ng[b].item()) == nb, (step, b)
            nxt.append(nb)
        t = nxt
    # the greedy loop as a captured graph reproduces the same tokens
    toks_g, _ = g.decode_greedy(list(range(batch)), t, 3)
    cur = list(t)
    for s_ in range(3):
        for b in range(batch):
            _, cur[b] = o.step_token(b, cur[b], fl)
        assert [int(v) for v in toks_g[s_].tolist()] == cur


def test_f16_config1_shape_prompt128_decode128(nnc):
    """The paper's F16 model at its own size: Qwen3-0.6B-shaped, binary16 weights and cache, a
    128-token prompt and 128 decode steps, teacher-forced on the oracle's tokens, then the
    free-running on-device loop (the launch configuration bench.py times)."""
    print("case: Qwen3-0.6B-shaped binary16 model, 128 + 128", flush=True)
    shape = synth.SHAPES["qwen3-0.6b-f16"]
    T, S = 128, 128
    blob = synth.make_blob(shape)
    g = nnc.Model(shape, blob, 1, T + S)
    o = oracle.from_shape(shape, blob, 1, T + S)
    fl = oracle_flags(shape)
    toks = synth.tokens(T, shape.vocab)
    lo, first = o.prefill(0, toks, fl)
    lg, ng = g.prefill(0, toks)
    err = float(np.abs(lg.double().cpu().numpy() - lo).max())
    print(f"  prompt last-position max abs err {err:.3e}, margin {top2_margin(lo):.3e}", flush=True)
    assert err <= F16_ABS and int(ng.item()) == first
    want, ties, max_err, min_margin = [], [], err, np.inf
    t = first
    for step in range(S):
        lo, nxt = o.step_token(0, t, fl)
        lg, ng = g.decode_step([0], [t])
        e = float(np.abs(lg[0].double().cpu().numpy() - lo).max())
        mg = top2_margin(lo)
        max_err, min_margin = max(max_err, e), min(min_margin, mg)
        assert e <= F16_ABS, (step, e)
        if int(ng.item()) != nxt:
            assert mg < 4 * e, (step, mg, e)
            ties.append(step)
        want.append(nxt)
        t = nxt
    print(f"  max abs err {max_err:.3e}; min top-2 margin {min_margin:.3e}; ties within error: {ties}", flush=True)
    assert not ties
    g.kv_reset(0)
    g.prefill(0, toks, want_logits=False)
    got, _ = g.decode_greedy([0], [first], S)
    assert np.array_equal(got.cpu().numpy()[:, 0], np.array(want))
