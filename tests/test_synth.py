"""Seeded input generator: determinism, distribution, blob layout."""
import numpy as np

import synth


def test_counter_based_and_order_free():
    a = synth.activations(4, 8, stream=3)
    b = synth.activations(4, 8, stream=3)
    assert np.array_equal(a, b)
    assert not np.array_equal(a, synth.activations(4, 8, stream=4))
    # element i is a function of (seed, tensor, i) alone: a later window matches
    lib = synth._load()
    whole = np.empty(100, np.float32)
    part = np.empty(10, np.float32)
    lib.synth_normal_f32(7, 5, 0, 100, 1.0, whole.ctypes.data)
    lib.synth_normal_f32(7, 5, 40, 10, 1.0, part.ctypes.data)
    assert np.array_equal(whole[40:50], part)


def test_mixer_matches_published_splitmix64_stream():
    # splitmix64 seeded with 0 yields this well-known first output; the generator
    # hashes key k as the splitmix64 output for state k, so raw(0, 0, 0) is it.
    assert synth.raw(0, 0, 0) == 0xE220A8397B1DCDAF


def test_normal_moments():
    x = synth.activations(1000, 1000, stream=9).astype(np.float64).ravel()
    assert abs(x.mean()) < 5e-3
    assert abs(x.std() - 1.0) < 5e-3
    assert abs((x ** 3).mean()) < 2e-2
    assert abs((x ** 4).mean() - 3.0) < 5e-2
    assert np.isfinite(x).all()


def test_tokens_uniform_in_range():
    t = synth.tokens(200000, 151936)
    assert t.min() >= 0 and t.max() < 151936
    assert abs(t.mean() / 151936 - 0.5) < 5e-3
    assert not np.array_equal(t[:100], synth.tokens(100, 151936, stream=1))


def test_blob_layout_and_sizes():
    s = synth.SHAPES["layer-0.6b-f32"]
    table, total = synth.blob_offsets(s)
    assert total == 4 * (15_728_640 + 2 * 1024 + 2 * 128)
    s1 = synth.SHAPES["qwen3-0.6b"]
    _, total1 = synth.blob_offsets(s1)
    matmul_params = 28 * 15_728_640 + 151936 * 1024
    assert matmul_params == 595_984_384
    assert total1 == 2 * matmul_params + 4 * (28 * (2 * 1024 + 256) + 1024)
    names = [n for n, _, _ in synth.blob_layout(s1)]
    assert names[0] == "embed" and names[-1] == "g_final"
    assert "lm_head" in [n for n, _, _ in synth.blob_layout(synth.SHAPES["qwen3-8b"])]


def test_bf16_blob_is_rounded_fp32_sample(tiny_shape):
    import torch
    sb = tiny_shape.scaled(dtype=synth.BF16)
    bf = synth.blob_tensor(sb, synth.make_blob(sb), "l0.wq")
    f32 = synth.blob_tensor(tiny_shape, synth.make_blob(tiny_shape), "l0.wq")
    want = torch.from_numpy(f32.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bf, want)
    g = synth.blob_tensor(sb, synth.make_blob(sb), "l1.g_post")
    assert g.dtype == np.float32 and np.all(g == 1.0)
    w = synth.bf16_bits_to_f32(bf).astype(np.float64)
    assert abs(w.std() - 0.02) < 2e-3


def test_f16_blob_is_rounded_fp32_sample(tiny_shape):
    sh = tiny_shape.scaled(dtype=synth.F16)
    h = synth.blob_tensor(sh, synth.make_blob(sh), "l0.wq")
    f32 = synth.blob_tensor(tiny_shape, synth.make_blob(tiny_shape), "l0.wq")
    assert np.array_equal(h, f32.astype(np.float16).view(np.uint16))     # numpy's cast: nearest even
    # small magnitudes (subnormal binary16 results) and the overflow edge go through the same store
    lib = synth._load()
    n = 4096
    for scale in (1e-6, 3e-5, 2e4):
        a = np.empty(n, np.float32)
        b = np.empty(n, np.uint16)
        lib.synth_normal_f32(5, 9, 0, n, scale, a.ctypes.data)
        lib.synth_normal_f16(5, 9, 0, n, scale, b.ctypes.data)
        with np.errstate(over="ignore"):
            assert np.array_equal(b, a.astype(np.float16).view(np.uint16)), scale
    w = synth.f16_bits_to_f32(h).astype(np.float64)
    assert abs(w.std() - 0.02) < 2e-3


def test_w8_blob_is_a_rowwise_quantised_sample(tiny_shape):
    """Weight-only 8-bit blobs: bytes + one scale per output row, next to the fp32 draw of the same
    (seed, tensor, index): scales have 8 significant bits, every row uses the full byte range, the
    stored weight is within half a step of the draw, embedding and gains are as in a bf16 blob."""
    s8 = tiny_shape.scaled(dtype=synth.W8)
    blob = synth.make_blob(s8)
    table, total = synth.blob_offsets(s8)
    assert blob.nbytes == total
    f32 = synth.make_blob(tiny_shape)
    for name in ("l0.wq", "l1.wdown", "l0.wgate"):
        q = synth.blob_tensor(s8, blob, name)
        sc = synth.blob_tensor(s8, blob, name + ".scale")
        w = synth.blob_tensor(tiny_shape, f32, name).astype(np.float64)
        assert q.dtype == np.int8 and sc.dtype == np.float32 and sc.shape == (q.shape[0],)
        assert np.all(sc.view(np.uint32) & 0xffff == 0) and np.all(sc > 0)        # bf16-representable
        assert np.abs(q.astype(np.int32)).max() <= 127
        assert np.all(np.abs(q.astype(np.int32)).max(axis=1) >= 126)            # scale = row maximum / 127, rounded up
        assert np.all(sc.astype(np.float64) * 127 >= np.abs(w).max(axis=1) - 1e-9)
        err = np.abs(q.astype(np.float64) * sc.astype(np.float64)[:, None] - w)
        assert np.all(err <= 0.5 * sc.astype(np.float64)[:, None] + 1e-8)        # nearest step (the fp32 draw is rounded)
    sb = tiny_shape.scaled(dtype=synth.BF16)
    assert np.array_equal(synth.blob_tensor(s8, blob, "embed"), synth.blob_tensor(sb, synth.make_blob(sb), "embed"))
    assert np.all(synth.blob_tensor(s8, blob, "l1.g_post") == 1.0)
