"""Pins for the oracle's building blocks: closed forms, invariants, brute force.

Each check is chosen so that a plausible slip (dropped term, wrong sign or index,
transposed operand, wrong scale) fails it.  None of them re-types the oracle's
own formula and compares the two.
"""
import math

import numpy as np
import pytest

import oracle

EPS = 1e-6
THETA = 1e6
rng = np.random.default_rng(20251221)


# ---- bf16 rounding -------------------------------------------------------------

def test_bf16_ties_go_to_even_and_exact_values_stay():
    assert oracle.bf16_round(1.0) == 1.0
    assert oracle.bf16_round(1.0 + 2 ** -7) == 1.0 + 2 ** -7          # representable
    assert oracle.bf16_round(1.0 + 2 ** -8) == 1.0                      # tie -> even (down)
    assert oracle.bf16_round(1.0 + 3 * 2 ** -8) == 1.0 + 2 ** -6        # tie -> even (up)
    assert oracle.bf16_round(1.0 + 2 ** -8 + 2 ** -30) == 1.0 + 2 ** -7  # just above the tie
    assert oracle.bf16_round(-(1.0 + 3 * 2 ** -8)) == -(1.0 + 2 ** -6)
    assert oracle.bf16_round(0.0) == 0.0
    assert oracle.bf16_round(2.0 ** -133) == 2.0 ** -133                # smallest subnormal
    assert oracle.bf16_round(2.0 ** -134) == 0.0                        # tie -> even (zero)
    assert math.isinf(oracle.bf16_round(3.4e38))


def test_bf16_matches_library_conversion_on_random_and_edge_floats():
    import torch
    bits = rng.integers(0, 2 ** 32, size=200000, dtype=np.uint64).astype(np.uint32)
    edge = np.array([0x3f808000, 0x3f818000, 0x3f807fff, 0x3f808001, 0x00000001, 0x00008000,
                     0x00018000, 0x7f7fffff, 0x80000000, 0x7f800000, 0xff800000], dtype=np.uint32)
    f = np.concatenate([bits, edge]).view(np.float32)
    f = f[~np.isnan(f)]
    want = torch.from_numpy(f.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.bf16_bits(v) for v in f], dtype=np.uint16)
    assert np.array_equal(got, want)


def test_bf16_error_at_most_half_ulp():
    x = rng.normal(size=2000)
    r = np.array([oracle.bf16_round(v) for v in x])
    ulp = 2.0 ** (np.floor(np.log2(np.abs(x))) - 7)
    assert np.all(np.abs(r - x) <= ulp / 2)


# ---- binary16 rounding (the paper's "F16") --------------------------------------------

def test_f16_ties_range_and_subnormals():
    assert oracle.f16_round(1.0) == 1.0
    assert oracle.f16_round(1.0 + 2 ** -10) == 1.0 + 2 ** -10           # representable
    assert oracle.f16_round(1.0 + 2 ** -11) == 1.0                       # tie -> even (down)
    assert oracle.f16_round(1.0 + 3 * 2 ** -11) == 1.0 + 2 ** -9         # tie -> even (up)
    assert oracle.f16_round(1.0 + 2 ** -11 + 2 ** -40) == 1.0 + 2 ** -10
    assert oracle.f16_round(-(1.0 + 3 * 2 ** -11)) == -(1.0 + 2 ** -9)
    assert oracle.f16_round(65504.0) == 65504.0                          # largest finite
    assert oracle.f16_round(65519.99) == 65504.0
    assert math.isinf(oracle.f16_round(65520.0))                         # tie -> even = overflow
    assert oracle.f16_round(2.0 ** -24) == 2.0 ** -24                    # smallest subnormal
    assert oracle.f16_round(2.0 ** -25) == 0.0                           # tie -> even (zero)
    assert oracle.f16_round(3 * 2.0 ** -25) == 2.0 ** -23                # tie -> even (up)
    assert oracle.f16_round(2.0 ** -14 + 2.0 ** -25) == 2.0 ** -14       # spacing 2^-24 at the bottom normal


def test_f16_matches_library_conversion_on_random_and_edge_floats():
    # numpy's float32 -> float16 cast is IEEE round-to-nearest-even: an independent implementation
    bits = rng.integers(0, 2 ** 32, size=200000, dtype=np.uint64).astype(np.uint32)
    near = (rng.normal(size=50000) * 0.02).astype(np.float32).view(np.uint32)   # the weights' range
    tiny = (rng.normal(size=20000) * 1e-6).astype(np.float32).view(np.uint32)   # subnormal results
    edge = np.array([0x3f801000, 0x3f803000, 0x3f800fff, 0x3f801001, 0x33000000, 0x33800000,
                     0x33c00000, 0x387fe000, 0x387ff000, 0x477fe000, 0x477fefff, 0x477ff000,
                     0x7f7fffff, 0x80000000, 0x7f800000, 0xff800000], dtype=np.uint32)
    f = np.concatenate([bits, near, tiny, edge]).view(np.float32)
    f = f[~np.isnan(f)]
    with np.errstate(over="ignore"):
        want = f.astype(np.float16).view(np.uint16)
    got = np.array([oracle.f16_bits(v) for v in f], dtype=np.uint16)
    assert np.array_equal(got, want)
    back = np.array([oracle.f16_round(float(v)) for v in f[:5000]])
    with np.errstate(over="ignore"):
        assert np.array_equal(back, f[:5000].astype(np.float16).astype(np.float64))


def test_matvec_f16_storage_is_widened_exactly():
    wf = np.concatenate([rng.normal(size=50) * 0.02, rng.normal(size=4) * 1e-6]).astype(np.float32).reshape(6, 9)
    wh = wf.astype(np.float16)                                            # includes subnormal entries
    assert np.any(np.abs(wh) < 2.0 ** -14)
    x = rng.normal(size=9)
    want = wh.astype(np.float64) @ x
    assert np.allclose(oracle.matvec(wh.view(np.uint16), x, oracle.F16), want, rtol=1e-14, atol=0)


# ---- matvec ----------------------------------------------------------------------

def test_matvec_against_naive_triple_loop():
    w = rng.normal(size=(3, 5)).astype(np.float32)
    x = rng.normal(size=5)
    want = [sum(float(w[r, k]) * x[k] for k in range(5)) for r in range(3)]
    assert np.allclose(oracle.matvec(w, x), want, rtol=1e-15, atol=0)


def test_matvec_identity_and_one_hot_select_rows_and_columns():
    n = 7
    x = rng.normal(size=n)
    assert np.array_equal(oracle.matvec(np.eye(n, dtype=np.float32), x), x)
    w = rng.normal(size=(4, n)).astype(np.float32)          # non-square: a transpose would fail
    e = np.zeros(n)
    e[2] = 1.0
    assert np.array_equal(oracle.matvec(w, e), w[:, 2].astype(np.float64))


def test_matvec_bf16_storage_is_widened_exactly():
    import torch
    wf = rng.normal(size=(6, 9)).astype(np.float32)
    wb = torch.from_numpy(wf).to(torch.bfloat16)
    bits = wb.view(torch.int16).numpy().view(np.uint16)
    x = rng.normal(size=9)
    want = wb.to(torch.float64).numpy() @ x
    assert np.allclose(oracle.matvec(bits, x, oracle.BF16), want, rtol=1e-14, atol=0)


# ---- RMSNorm ---------------------------------------------------------------------

def test_rmsnorm_constant_vector_closed_form():
    c, n = 3.0, 16
    g = np.linspace(0.5, 2.0, n)
    out = oracle.rmsnorm(np.full(n, c), g, EPS)
    assert np.allclose(out, c / math.sqrt(c * c + EPS) * g, rtol=1e-15)


def test_rmsnorm_unit_rms_before_gain_and_eps_inside_sqrt():
    x = rng.normal(size=128)
    ms = float(np.mean(x * x))
    out = oracle.rmsnorm(x, None, EPS)
    assert math.isclose(math.sqrt(np.mean(out * out)), math.sqrt(ms / (ms + EPS)), rel_tol=1e-14)
    # with a large eps the placement (inside the root, added to the MEAN) is visible
    out2 = oracle.rmsnorm(x, None, 0.5)
    assert math.isclose(math.sqrt(np.mean(out2 * out2)), math.sqrt(ms / (ms + 0.5)), rel_tol=1e-14)


def test_rmsnorm_scale_invariant_zero_safe_and_gain_is_plain_elementwise():
    x = rng.normal(size=64)
    assert np.allclose(oracle.rmsnorm(37.0 * x, None, EPS), oracle.rmsnorm(x, None, EPS), rtol=1e-5)
    z = oracle.rmsnorm(np.zeros(8), np.ones(8), EPS)
    assert np.all(z == 0.0)
    g = np.zeros(64)
    g[5] = 2.0                                    # (1 + g) style gain would leave other entries alive
    out = oracle.rmsnorm(x, g, EPS)
    base = oracle.rmsnorm(x, None, EPS)
    assert out[5] == 2.0 * base[5] and np.count_nonzero(out) == 1


# ---- RoPE ------------------------------------------------------------------------

def test_rope_position_zero_is_identity_bit_exact():
    u = rng.normal(size=128)
    assert np.array_equal(oracle.rope(u, 0, THETA), u)


def test_rope_preserves_pair_and_head_norms():
    d = 128
    u = rng.normal(size=d)
    r = oracle.rope(u, 4223, THETA)
    assert np.allclose(u[:64] ** 2 + u[64:] ** 2, r[:64] ** 2 + r[64:] ** 2, rtol=1e-13)
    assert math.isclose(np.linalg.norm(u), np.linalg.norm(r), rel_tol=1e-14)


def test_rope_closed_form_first_and_last_pair():
    d, p = 128, 7
    u = np.zeros(d)
    u[0] = 1.0                                        # pair 0 = (index 0, index d/2), frequency 1
    r = oracle.rope(u, p, THETA)
    assert math.isclose(r[0], math.cos(p), rel_tol=1e-15)
    assert math.isclose(r[64], math.sin(p), rel_tol=1e-15)
    assert np.count_nonzero(r) == 2
    u = np.zeros(d)
    u[127] = 1.0                                      # second element of the last pair (63, 127)
    p = 100000
    phi = p * THETA ** (-(d - 2) / d)
    r = oracle.rope(u, p, THETA)
    assert math.isclose(r[63], -math.sin(phi), rel_tol=1e-12)
    assert math.isclose(r[127], math.cos(phi), rel_tol=1e-12)


def test_rope_relative_position_and_additivity():
    q, k = rng.normal(size=128), rng.normal(size=128)
    m, n = 911, 377
    lhs = oracle.rope(q, m, THETA) @ oracle.rope(k, n, THETA)
    rhs = oracle.rope(q, m - n, THETA) @ k
    assert math.isclose(lhs, rhs, rel_tol=1e-10, abs_tol=1e-10)
    twice = oracle.rope(oracle.rope(q, m, THETA), n, THETA)
    assert np.allclose(twice, oracle.rope(q, m + n, THETA), rtol=0, atol=1e-10)


# ---- softmax ---------------------------------------------------------------------

def test_softmax_closed_forms():
    s = rng.normal(size=33) * 3
    w = oracle.softmax(s)
    assert abs(w.sum() - 1.0) <= 1e-15 * 33
    assert np.allclose(oracle.softmax(s + 123.0), w, rtol=1e-12)
    assert oracle.softmax([4.2])[0] == 1.0
    assert np.array_equal(oracle.softmax([1.5, 1.5]), [0.5, 0.5])
    big = oracle.softmax([1e4, -1e4, 1e4 - math.log(3.0)])
    assert np.isfinite(big).all()
    assert np.allclose(big, [0.75, 0.0, 0.25], atol=1e-12)
    assert np.allclose(oracle.softmax([0.0, math.log(2.0)]), [1 / 3, 2 / 3], rtol=1e-15)


# ---- attention -------------------------------------------------------------------

def test_attend_scale_is_one_over_sqrt_d():
    d = 16
    q = np.zeros(d)
    q[0] = math.sqrt(d) * math.log(2.0)
    keys = np.zeros((2, d))
    keys[0, 0] = 1.0                                   # scores (ln 2, 0) -> weights (2/3, 1/3)
    vals = np.zeros((2, d))
    vals[0, 3], vals[1, 3] = 3.0, 6.0
    out = oracle.attend(q, keys, vals)
    assert math.isclose(out[3], 4.0, rel_tol=1e-14)
    assert np.count_nonzero(out) == 1


def test_attend_brute_force_four_tokens():
    d, n = 8, 4
    Q, K, V = rng.normal(size=(n, d)), rng.normal(size=(n, d)), rng.normal(size=(n, d))
    S = np.full((n, n), -np.inf)
    for i in range(n):
        for j in range(i + 1):                      # causal mask j <= i
            S[i, j] = sum(Q[i, t] * K[j, t] for t in range(d)) / math.sqrt(d)
    P = np.exp(S - S.max(axis=1, keepdims=True))
    P /= P.sum(axis=1, keepdims=True)
    want = P @ V
    for i in range(n):
        got = oracle.attend(Q[i], K[: i + 1], V[: i + 1])
        assert np.allclose(got, want[i], rtol=1e-13, atol=1e-15)


def test_attend_single_key_returns_its_value_and_equal_keys_average():
    d = 8
    q = rng.normal(size=d)
    v = rng.normal(size=(1, d))
    assert np.allclose(oracle.attend(q, rng.normal(size=(1, d)), v), v[0], rtol=1e-15)
    k = np.tile(rng.normal(size=d), (5, 1))
    vals = rng.normal(size=(5, d))
    assert np.allclose(oracle.attend(q, k, vals), vals.mean(axis=0), rtol=1e-13)


def test_attend_rounded_weights_variant():
    d = 4
    q = np.array([2.0 * math.log(3.0), 0, 0, 0])       # scores (ln 3, 0) after the 1/2 scale
    keys = np.array([[1.0, 0, 0, 0], [0.0, 0, 0, 0]])
    vals = np.array([[1.0, 0, 0, 0], [0.0, 1.0, 0, 0]])
    # un-normalised weights (1, 1/3); 1/3 rounds to bf16 0.333984375
    third = oracle.bf16_round(1.0 / 3.0)
    assert third == 0.333984375
    out = oracle.attend(q, keys, vals, round_p=1)
    assert np.allclose(out[:2], [1 / (1 + third), third / (1 + third)], rtol=1e-14)
    # binary16: 1/3 rounds to 0.333251953125
    third = oracle.f16_round(1.0 / 3.0)
    assert third == 0.333251953125
    out = oracle.attend(q, keys, vals, round_p=2)
    assert np.allclose(out[:2], [1 / (1 + third), third / (1 + third)], rtol=1e-14)


# ---- SwiGLU pieces, argmax ----------------------------------------------------------

def test_silu_values():
    assert oracle.silu(0.0) == 0.0
    assert math.isclose(oracle.silu(1.0), 1.0 / (1.0 + math.exp(-1.0)), rel_tol=1e-16)
    assert math.isclose(oracle.silu(40.0), 40.0, rel_tol=1e-15)
    assert abs(oracle.silu(-40.0)) < 1e-15
    assert oracle.silu(-800.0) == 0.0 or abs(oracle.silu(-800.0)) < 1e-300   # no NaN from exp overflow
    assert math.isclose(oracle.silu(-1.0), -1.0 / (1.0 + math.e), rel_tol=1e-15)


def test_argmax_lowest_index_wins_and_nan_never_does():
    assert oracle.argmax([0.0, 0.0, 0.0]) == 0
    assert oracle.argmax([1.0, 5.0, 5.0, 2.0]) == 1
    assert oracle.argmax([-3.0, -1.0, -2.0]) == 1
    assert oracle.argmax([1.0, float("nan"), 3.0]) == -1
