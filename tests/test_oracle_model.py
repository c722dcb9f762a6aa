"""Pins for the oracle's whole forward pass: structure, cache, conventions.

The conventions the paper leaves open (RoPE pairing, norm-then-RoPE order, GQA
grouping, gain form, SwiGLU branch, softmax scale, tied head) are pinned by a
black-box comparison with the Qwen3 model class of the installed `transformers`
package, built offline from a config, loaded with the oracle's own weights and
run in fp64.  That library is only ever used here, as a test.
"""
import math

import numpy as np
import pytest

import oracle
import synth


def _mk(shape, blob, max_batch=2, max_seq=16):
    return oracle.from_shape(shape, blob, max_batch, max_seq)


def _set(shape, blob, name, value):
    t = synth.blob_tensor(shape, blob, name)
    t[...] = value


def test_blob_size_is_checked(tiny_shape):
    blob = synth.make_blob(tiny_shape)
    with pytest.raises(ValueError):
        _mk(tiny_shape, blob[:-4])


def test_zero_output_projections_make_the_layer_an_identity(tiny_shape):
    s = tiny_shape.scaled(has_embed_and_head=False, tied_lm_head=False, vocab=0, n_layers=1)
    blob = synth.make_blob(s, gain_jitter=0.1)
    _set(s, blob, "l0.wo", 0.0)
    _set(s, blob, "l0.wdown", 0.0)
    m = _mk(s, blob)
    x = synth.activations(3, s.hidden).astype(np.float64)
    for t in range(3):
        assert np.array_equal(m.step_hidden(0, x[t]), x[t])


def test_all_zero_weights_give_zero_logits_and_token_zero(tiny_shape):
    blob = synth.make_blob(tiny_shape)
    for name, _, is_gain in synth.blob_layout(tiny_shape):
        if not is_gain:
            _set(tiny_shape, blob, name, 0.0)
    m = _mk(tiny_shape, blob)
    logits, nxt = m.step_token(0, 7)
    assert np.all(logits == 0.0) and nxt == 0


def test_zero_layer_model_is_embedding_norm_head_closed_form(tiny_shape):
    s = tiny_shape.scaled(n_layers=0)
    blob = synth.make_blob(s, weight_std=1.0, gain_jitter=0.2)
    E = synth.blob_tensor(s, blob, "embed").astype(np.float64)
    g = synth.blob_tensor(s, blob, "g_final").astype(np.float64)
    m = _mk(s, blob)
    t = 11
    xn = E[t] / math.sqrt(np.mean(E[t] ** 2) + s.rms_eps) * g
    logits, nxt = m.step_token(0, t)
    assert np.allclose(logits, E @ xn, rtol=1e-13)
    assert nxt == int(np.argmax(E @ xn))


def test_untied_head_reads_its_own_matrix(tiny_shape):
    s = tiny_shape.scaled(n_layers=0, tied_lm_head=False)
    blob = synth.make_blob(s, weight_std=1.0)
    E = synth.blob_tensor(s, blob, "embed").astype(np.float64)
    W = synth.blob_tensor(s, blob, "lm_head").astype(np.float64)
    m = _mk(s, blob)
    xn = E[3] / math.sqrt(np.mean(E[3] ** 2) + s.rms_eps)
    logits, _ = m.step_token(0, 3)
    assert np.allclose(logits, W @ xn, rtol=1e-13)


def test_first_position_attention_output_is_the_value_row_of_its_group(tiny_shape):
    # at position 0 softmax has one entry, so o_a = v_{a // G}; with Wo chosen to copy
    # one q head's slot into the residual, the GQA mapping and the V path are visible.
    s = tiny_shape.scaled(has_embed_and_head=False, tied_lm_head=False, vocab=0, n_layers=1)
    blob = synth.make_blob(s, weight_std=0.3, gain_jitter=0.1)
    _set(s, blob, "l0.wdown", 0.0)
    d, H, G = s.head_dim, s.hidden, s.n_q_heads // s.n_kv_heads
    wo = synth.blob_tensor(s, blob, "l0.wo")
    wv = synth.blob_tensor(s, blob, "l0.wv").astype(np.float64)
    g_in = synth.blob_tensor(s, blob, "l0.g_in").astype(np.float64)
    x = synth.activations(1, H)[0].astype(np.float64)
    h = x / math.sqrt(np.mean(x * x) + s.rms_eps) * g_in
    v = wv @ h
    for a in range(s.n_q_heads):
        wo[...] = 0.0
        for i in range(d):
            wo[i, a * d + i] = 1.0                  # residual[i] += o_a[i]
        m = _mk(s, blob)
        y = m.step_hidden(0, x)
        b = a // G
        assert np.allclose(y[:d] - x[:d], v[b * d:(b + 1) * d], rtol=1e-12, atol=1e-14)
        assert np.array_equal(y[d:], x[d:])


def test_prefill_equals_incremental_decode_and_reset_replays(tiny_shape):
    blob = synth.make_blob(tiny_shape, weight_std=0.2, gain_jitter=0.1)
    toks = synth.tokens(9, tiny_shape.vocab)
    m = _mk(tiny_shape, blob)
    lp, np_ = m.prefill(0, toks)
    for t in toks[:-1]:
        m.step_token(1, t, want_logits=False)
    ls, ns = m.step_token(1, toks[-1])
    assert np.array_equal(lp, ls) and np_ == ns
    assert m.slot_len(0) == 9 and m.slot_len(1) == 9
    m.kv_reset(0)
    assert m.slot_len(0) == 0 and m.slot_len(1) == 9
    lr, _ = m.prefill(0, toks)
    assert np.array_equal(lr, lp)


def test_causality_and_slot_independence(tiny_shape):
    blob = synth.make_blob(tiny_shape, weight_std=0.2)
    a = synth.tokens(6, tiny_shape.vocab)
    b = a.copy()
    b[4:] = (b[4:] + 1) % tiny_shape.vocab          # change only later tokens
    m = _mk(tiny_shape, blob)
    outs_a = [m.step_token(0, t)[0] for t in a]
    outs_b = [m.step_token(1, t)[0] for t in b]
    for i in range(4):
        assert np.array_equal(outs_a[i], outs_b[i])
    assert not np.array_equal(outs_a[4], outs_b[4])
    # slot 1 was interleaved with nothing else; rerun slot 0's sequence alone
    m2 = _mk(tiny_shape, blob)
    for i, t in enumerate(a):
        assert np.array_equal(m2.step_token(0, t)[0], outs_a[i])


def test_kv_capacity_is_an_error_not_a_wraparound(tiny_shape):
    m = _mk(tiny_shape, synth.make_blob(tiny_shape), max_batch=1, max_seq=2)
    m.step_token(0, 1)
    m.step_token(0, 2)
    with pytest.raises(RuntimeError):
        m.step_token(0, 3)


def test_gqa_equals_mha_with_repeated_kv_heads(tiny_shape):
    s = tiny_shape
    blob = synth.make_blob(s, weight_std=0.2, gain_jitter=0.1)
    G, d = s.n_q_heads // s.n_kv_heads, s.head_dim
    mha = s.scaled(n_kv_heads=s.n_q_heads)
    blob2 = synth.make_blob(mha)
    for name, _, _ in synth.blob_layout(s):
        src = synth.blob_tensor(s, blob, name)
        dst = synth.blob_tensor(mha, blob2, name)
        if name.endswith(".wk") or name.endswith(".wv"):
            src = src.reshape(s.n_kv_heads, d, s.hidden)
            dst[...] = np.repeat(src, G, axis=0).reshape(dst.shape)   # contiguous groups
        else:
            dst[...] = src
    toks = synth.tokens(5, s.vocab)
    la, _ = _mk(s, blob).prefill(0, toks)
    lb, _ = _mk(mha, blob2).prefill(0, toks)
    assert np.allclose(la, lb, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("fmt", ["f32", "w8"])
def test_conventions_against_library_qwen3_in_fp64(tiny_shape, fmt):
    """fmt w8: the same cross-check on a weight-only 8-bit blob.  The library model gets
    scale[row] * byte taken from the blob through the generator's offset table (not through the
    oracle's own parser), so a misplaced scale, a scale applied per column, or matrices read in
    the wrong order in the oracle's widening would show as a disagreement."""
    torch = pytest.importorskip("torch")
    tr = pytest.importorskip("transformers")
    try:
        from transformers import Qwen3Config, Qwen3ForCausalLM
    except Exception as e:  # pragma: no cover
        pytest.skip(f"library Qwen3 class unavailable: {e}")
    s = tiny_shape if fmt == "f32" else tiny_shape.scaled(dtype=synth.W8)
    blob = synth.make_blob(s, weight_std=0.25, gain_jitter=0.2)
    cfg = Qwen3Config(vocab_size=s.vocab, hidden_size=s.hidden, intermediate_size=s.ffn,
                      num_hidden_layers=s.n_layers, num_attention_heads=s.n_q_heads,
                      num_key_value_heads=s.n_kv_heads, head_dim=s.head_dim,
                      rms_norm_eps=s.rms_eps, rope_theta=s.rope_theta, tie_word_embeddings=True,
                      attention_bias=False, max_position_embeddings=64, use_sliding_window=False,
                      attn_implementation="eager")
    if getattr(cfg, "rope_parameters", None) is not None:
        cfg.rope_parameters = {"rope_type": "default", "rope_theta": s.rope_theta}
    model = Qwen3ForCausalLM(cfg).to(torch.float64).eval()
    def get(n):
        t = synth.blob_tensor(s, blob, n)
        if t.dtype == np.int8:
            return torch.from_numpy(t.astype(np.float64) * synth.blob_tensor(s, blob, n + ".scale").astype(np.float64)[:, None])
        if t.dtype == np.uint16:
            return torch.from_numpy(synth.bf16_bits_to_f32(t).astype(np.float64))
        return torch.from_numpy(t.astype(np.float64))
    sd = {"model.embed_tokens.weight": get("embed"), "model.norm.weight": get("g_final"),
          "lm_head.weight": get("embed")}
    names = {"g_in": "input_layernorm.weight", "wq": "self_attn.q_proj.weight",
             "wk": "self_attn.k_proj.weight", "wv": "self_attn.v_proj.weight",
             "g_q": "self_attn.q_norm.weight", "g_k": "self_attn.k_norm.weight",
             "wo": "self_attn.o_proj.weight", "g_post": "post_attention_layernorm.weight",
             "wgate": "mlp.gate_proj.weight", "wup": "mlp.up_proj.weight",
             "wdown": "mlp.down_proj.weight"}
    for l in range(s.n_layers):
        for k, v in names.items():
            sd[f"model.layers.{l}.{v}"] = get(f"l{l}.{k}")
    missing, unexpected = model.load_state_dict(sd, strict=False)
    assert not unexpected and all("rotary" in k or "inv_freq" in k for k in missing), (missing, unexpected)
    # the rotary table of the library model is fp32-derived; rebuild it in fp64
    rot = model.model.rotary_emb
    inv = 1.0 / (s.rope_theta ** (torch.arange(0, s.head_dim, 2, dtype=torch.float64) / s.head_dim))
    rot.inv_freq = inv
    if hasattr(rot, "original_inv_freq"):
        rot.original_inv_freq = inv
    toks = synth.tokens(12, s.vocab)
    with torch.no_grad():
        want = model(torch.from_numpy(toks.astype(np.int64))[None]).logits[0].numpy()
    m = _mk(s, blob)
    for i, t in enumerate(toks):
        got, nxt = m.step_token(0, t)
        # the library computes angles/cos/sin through fp32 autocast-free paths of its own;
        # agreement is to ~1e-6, far below what any convention change would produce
        assert np.allclose(got, want[i], rtol=0, atol=2e-5 * np.abs(want[i]).max()), i
        assert nxt == int(np.argmax(want[i]))
    assert np.abs(want).max() > 0.1                       # the comparison is not vacuous


# ---- rounding points (flags) -------------------------------------------------------
#
# Every rounding flag is pinned by making ONE rounded vector observable through selector
# weights (rows of the identity) on a one-layer hidden-state model, and comparing with a value
# built from the closed-form RMSNorm, a numpy matrix product and the separately pinned scalar
# rounding function.  Each probe also shows that the plausible mistakes (rounding dropped,
# rounding at the neighbouring point instead) would give a different value.

FORMATS = [("bf16", 0), ("f16", oracle.ROUND_F16)]


def _rnd(fmt_flag):
    f = oracle.f16_round if fmt_flag else oracle.bf16_round
    return lambda a: np.array([f(float(v)) for v in np.ravel(a)]).reshape(np.shape(a))


def _layer_model(tiny_shape, **zero):
    s = tiny_shape.scaled(has_embed_and_head=False, tied_lm_head=False, vocab=0, n_layers=1)
    blob = synth.make_blob(s, weight_std=0.3, gain_jitter=0.1)
    return s, blob


def _selector(w, col0=0):
    """w[i, col0 + i] = 1, everything else 0: y = W x copies x[col0 : col0 + rows]."""
    w[...] = 0.0
    for i in range(w.shape[0]):
        if col0 + i < w.shape[1]:
            w[i, col0 + i] = 1.0


def _norm(x, g, eps):
    return x / math.sqrt(np.mean(x * x) + eps) * g


@pytest.mark.parametrize("fmt,ff", FORMATS)
def test_round_kv_flag_stores_rounded_values_of_the_exact_rows(tiny_shape, fmt, ff):
    blob = synth.make_blob(tiny_shape, weight_std=0.2)
    toks = synth.tokens(3, tiny_shape.vocab)
    rnd = _rnd(ff)
    exact, rounded = _mk(tiny_shape, blob), _mk(tiny_shape, blob)
    exact.step_token(0, toks[0], want_logits=False)
    rounded.step_token(0, toks[0], flags=oracle.ROUND_KV | ff, want_logits=False)
    for which in (0, 1):
        e = exact.kv_rows(0, 0, which)[0]            # layer 0, position 0 depends on no cache
        r = rounded.kv_rows(0, 0, which)[0]
        assert np.array_equal(r, rnd(e))
        assert np.any(r != e)


@pytest.mark.parametrize("fmt,ff", FORMATS)
def test_round_gemm_in_rounds_the_normed_input_of_the_qkv_projections(tiny_shape, fmt, ff):
    # Wv = rows of the identity: the cached V row IS the projection's input vector
    s, blob = _layer_model(tiny_shape)
    _selector(synth.blob_tensor(s, blob, "l0.wv"))
    g_in = synth.blob_tensor(s, blob, "l0.g_in").astype(np.float64)
    x = synth.activations(1, s.hidden)[0].astype(np.float64)
    h = _norm(x, g_in, s.rms_eps)
    m = _mk(s, blob)
    m.step_hidden(0, x, flags=oracle.ROUND_GEMM_IN | ff)
    m.step_hidden(1, x, flags=0)
    want = _rnd(ff)(h[:s.dkv])
    assert np.array_equal(m.kv_rows(0, 0, 1)[0], want)
    assert np.allclose(m.kv_rows(0, 1, 1)[0], h[:s.dkv], rtol=1e-14) and np.any(want != h[:s.dkv])


@pytest.mark.parametrize("fmt,ff", FORMATS)
def test_round_gemm_in_rounds_the_attention_output_before_the_o_projection(tiny_shape, fmt, ff):
    # position 0: o_a = v_{a // G}; Wo copies head a into the residual; Wdown = 0
    s, blob = _layer_model(tiny_shape)
    _set(s, blob, "l0.wdown", 0.0)
    d, G = s.head_dim, s.n_q_heads // s.n_kv_heads
    rnd = _rnd(ff)
    wv = synth.blob_tensor(s, blob, "l0.wv").astype(np.float64)
    g_in = synth.blob_tensor(s, blob, "l0.g_in").astype(np.float64)
    x = synth.activations(1, s.hidden)[0].astype(np.float64)
    v = wv @ rnd(_norm(x, g_in, s.rms_eps))           # the projection input is rounded too
    a = 3
    _selector(synth.blob_tensor(s, blob, "l0.wo")[:d], col0=a * d)
    synth.blob_tensor(s, blob, "l0.wo")[d:] = 0.0
    m = _mk(s, blob)
    y = m.step_hidden(0, x, flags=oracle.ROUND_GEMM_IN | ff)
    vb = v[(a // G) * d:(a // G + 1) * d]
    want = rnd(vb)
    # the residual add happens in fp64: y - x loses the bits below ulp(x)
    assert np.allclose(y[:d] - x[:d], want, rtol=0, atol=1e-14)
    assert np.abs(want - vb).max() > 1e-6             # an unrounded o would be off by far more than 1e-14


@pytest.mark.parametrize("fmt,ff", FORMATS)
def test_round_gemm_in_rounds_the_swiglu_product_once_after_multiplying(tiny_shape, fmt, ff):
    # Wo = 0 (attention adds nothing), Wdown copies act[0:H] into the residual
    s, blob = _layer_model(tiny_shape)
    _set(s, blob, "l0.wo", 0.0)
    _selector(synth.blob_tensor(s, blob, "l0.wdown"))
    rnd = _rnd(ff)
    H = s.hidden
    wg = synth.blob_tensor(s, blob, "l0.wgate").astype(np.float64)
    wu = synth.blob_tensor(s, blob, "l0.wup").astype(np.float64)
    g_post = synth.blob_tensor(s, blob, "l0.g_post").astype(np.float64)
    x = synth.activations(1, H, stream=2)[0].astype(np.float64)
    h2 = _norm(x, g_post, s.rms_eps)
    silu = lambda z: z / (1.0 + np.exp(-z))
    gate, up = wg @ rnd(h2), wu @ rnd(h2)
    want = rnd(silu(gate) * up)[:H]
    m = _mk(s, blob)
    y = m.step_hidden(0, x, flags=oracle.ROUND_GEMM_IN | ff)
    assert np.allclose(y - x, want, rtol=0, atol=1e-14)
    # the mistakes this must catch are visible at this tolerance:
    before = (rnd(silu(gate)) * rnd(up))[:H]                              # rounded before the product
    unrounded_h2 = rnd(silu(wg @ h2) * (wu @ h2))[:H]                     # second norm's rounding dropped
    no_act = (silu(gate) * up)[:H]                                        # act rounding dropped
    for wrong in (before, unrounded_h2, no_act):
        assert np.abs(wrong - want).max() > 1e-6


@pytest.mark.parametrize("fmt,ff", FORMATS)
def test_round_attn_qp_rounds_the_rotated_query_and_the_unnormalised_weights(tiny_shape, fmt, ff):
    # two cached positions; K / V rows are read back from the cache (no ORC_ROUND_KV: exact),
    # the rotated query is rebuilt from the pinned building blocks, the head's output is made
    # visible by a selector Wo with Wdown = 0
    s, blob = _layer_model(tiny_shape)
    _set(s, blob, "l0.wdown", 0.0)
    d, G, H = s.head_dim, s.n_q_heads // s.n_kv_heads, s.hidden
    rnd = _rnd(ff)
    a = 2
    b = a // G
    wo = synth.blob_tensor(s, blob, "l0.wo")
    _selector(wo[:d], col0=a * d)
    wo[d:] = 0.0
    wq = synth.blob_tensor(s, blob, "l0.wq").astype(np.float64)
    g_in = synth.blob_tensor(s, blob, "l0.g_in").astype(np.float64)
    synth.blob_tensor(s, blob, "l0.g_q")[...] *= 3.0    # wider scores: the query's rounding moves the weights
    g_q = synth.blob_tensor(s, blob, "l0.g_q").astype(np.float64)
    xs = 4.0 * synth.activations(2, H, stream=4).astype(np.float64)
    m = _mk(s, blob)
    fl = oracle.ROUND_ATTN_QP | ff
    y0 = m.step_hidden(0, xs[0], flags=fl)
    # the second input does not depend on the first output here (hidden-state model)
    y1 = m.step_hidden(0, xs[1], flags=fl)
    K = m.kv_rows(0, 0, 0)[:, b * d:(b + 1) * d]
    V = m.kv_rows(0, 0, 1)[:, b * d:(b + 1) * d]
    q = (wq @ _norm(xs[1], g_in, s.rms_eps))[a * d:(a + 1) * d]
    qt = oracle.rope(oracle.rmsnorm(q, g_q, s.rms_eps), 1, s.rope_theta)

    def attn(qv, round_w):
        sc = np.array([qv @ K[0], qv @ K[1]]) / math.sqrt(d)
        w = np.exp(sc - sc.max())
        if round_w:
            w = rnd(w)
        return (w[0] * V[0] + w[1] * V[1]) / (w[0] + w[1])

    want = attn(rnd(qt), True)
    assert np.allclose(y1[:d] - xs[1][:d], want, rtol=0, atol=1e-13)
    for wrong in (attn(qt, True), attn(rnd(qt), False), attn(qt, False)):
        assert np.abs(wrong - want).max() > 1e-7      # a million times the tolerance above
    # the query must not be rounded in the cache-facing path of K: rows are exact
    exact = _mk(s, blob)
    exact.step_hidden(0, xs[0])
    assert np.array_equal(exact.kv_rows(0, 0, 0)[0], m.kv_rows(0, 0, 0)[0])
    assert np.isfinite(y0).all()


@pytest.mark.parametrize("fmt,ff", FORMATS)
def test_round_head_in_needs_both_flags_and_rounds_the_final_norm_output(tiny_shape, fmt, ff):
    s = tiny_shape.scaled(n_layers=0)
    blob = synth.make_blob(s, weight_std=1.0, gain_jitter=0.2)
    E = synth.blob_tensor(s, blob, "embed").astype(np.float64)
    g = synth.blob_tensor(s, blob, "g_final").astype(np.float64)
    t = 17
    xn = _norm(E[t], g, s.rms_eps)
    m = _mk(s, blob)
    both, _ = m.step_token(0, t, flags=oracle.ROUND_GEMM_IN | oracle.ROUND_HEAD_IN | ff)
    only_in, _ = m.step_token(0, t, flags=oracle.ROUND_GEMM_IN | ff)
    only_head, _ = m.step_token(0, t, flags=oracle.ROUND_HEAD_IN | ff)
    assert np.allclose(both, E @ _rnd(ff)(xn), rtol=1e-13, atol=1e-13)
    assert np.allclose(only_in, E @ xn, rtol=1e-13, atol=1e-13)
    assert np.allclose(only_head, E @ xn, rtol=1e-13, atol=1e-13)
    assert np.abs(both - only_in).max() > 1e-4


def test_f16_blob_model_equals_fp32_model_of_the_widened_weights(tiny_shape):
    # the 16-bit storage formats are only a widening step: a binary16 blob gives exactly the
    # logits of an fp32 blob that holds the same values
    sh = tiny_shape.scaled(dtype=synth.F16)
    bh = synth.make_blob(sh, weight_std=0.2, gain_jitter=0.1)
    bf = synth.make_blob(tiny_shape, weight_std=0.2, gain_jitter=0.1)
    for name, _, is_gain in synth.blob_layout(sh):
        src = synth.blob_tensor(sh, bh, name)
        synth.blob_tensor(tiny_shape, bf, name)[...] = src if is_gain else synth.f16_bits_to_f32(src)
    toks = synth.tokens(5, sh.vocab)
    la, na = _mk(sh, bh).prefill(0, toks)
    lb, nb = _mk(tiny_shape, bf).prefill(0, toks)
    assert np.array_equal(la, lb) and na == nb
