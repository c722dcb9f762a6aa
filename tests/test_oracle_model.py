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


def test_conventions_against_library_qwen3_in_fp64(tiny_shape):
    torch = pytest.importorskip("torch")
    tr = pytest.importorskip("transformers")
    try:
        from transformers import Qwen3Config, Qwen3ForCausalLM
    except Exception as e:  # pragma: no cover
        pytest.skip(f"library Qwen3 class unavailable: {e}")
    s = tiny_shape
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
    get = lambda n: torch.from_numpy(synth.blob_tensor(s, blob, n).astype(np.float64))
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


def test_round_kv_flag_stores_bf16_values_of_the_exact_rows(tiny_shape):
    blob = synth.make_blob(tiny_shape, weight_std=0.2)
    toks = synth.tokens(3, tiny_shape.vocab)
    exact, rnd = _mk(tiny_shape, blob), _mk(tiny_shape, blob)
    exact.step_token(0, toks[0], want_logits=False)
    rnd.step_token(0, toks[0], flags=oracle.ROUND_KV, want_logits=False)
    for which in (0, 1):
        e = exact.kv_rows(0, 0, which)[0]            # layer 0, position 0 depends on no cache
        r = rnd.kv_rows(0, 0, which)[0]
        assert np.array_equal(r, [oracle.bf16_round(v) for v in e])
        assert np.any(r != e)


def test_round_gemm_in_flag_is_a_small_perturbation(tiny_shape):
    blob = synth.make_blob(tiny_shape, weight_std=0.2)
    toks = synth.tokens(6, tiny_shape.vocab)
    a, _ = _mk(tiny_shape, blob).prefill(0, toks)
    b, _ = _mk(tiny_shape, blob).prefill(0, toks, flags=oracle.ROUND_GEMM_IN | oracle.ROUND_HEAD_IN)
    c, _ = _mk(tiny_shape, blob).prefill(0, toks, flags=oracle.ROUND_GEMM_IN)
    err = np.abs(a - b).max() / np.abs(a).max()
    assert 1e-5 < err < 3e-2
    assert not np.array_equal(b, c)
