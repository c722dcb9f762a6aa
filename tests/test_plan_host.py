"""The analytic tile chooser (host code, no GPU): constraints, objective, and that it lands on
the choices that were found by hand and measured on the large shapes.

Model after the paper's parametric optimisation (Section 3.2.2): tile variables, capacity
constraints per storage level, minimise max(T_mem, T_comp) + launch and epilogue time.
"""
import pytest

from paper_2512_21571_amd import binding as nnc

STORE, RESID, SWIGLU = 0, 1, 2
SHAPES = {  # hidden, Dq, Dkv, ffn
    "0.6b": (1024, 2048, 1024, 3072), "1.7b": (2048, 2048, 1024, 6144),
    "4b": (2560, 4096, 1024, 9728), "8b": (4096, 4096, 1024, 12288)}
V = 151936


def _gemms(name):
    H, Dq, Dkv, F = SHAPES[name]
    return {"qkv": (Dq + 2 * Dkv, H, STORE), "o": (H, Dq, RESID), "gate_up": (2 * F, H, SWIGLU), "down": (H, F, RESID)}


def test_capacity_constraints_rule_out_what_does_not_fit():
    p = nnc.plan_prefill_gemm(24576, 4096, 4080, 1, SWIGLU)
    # 256 x 256 with two workgroups per CU: 3 stages x 32 KiB x 2 > 160 KiB, and 384 registers per
    # wave; with one workgroup per CU it fits (the accumulators in the accumulation registers)
    assert p.candidates == 8 and p.rejected_by_capacity == 1
    assert (p.tile_rows, p.tile_cols) == (256, 256)


B, M = (256, 256), (192, 256)     # the two tiles of one workgroup per CU


@pytest.mark.parametrize("name,tokens,want", [
    # the block tiles measured best (or within 5 % of the best) at the benchmark shapes: rows of a tile
    # of 128 operand columns, or one of the two 256-column tiles
    ("8b", 4080, {"qkv": M, "o": B, "gate_up": B, "down": B}),
    ("8b", 2032, {"qkv": M, "o": 128, "gate_up": B, "down": 128}),
    ("4b", 4080, {"qkv": M, "o": M, "gate_up": B, "down": M}),
    ("4b", 2032, {"qkv": M, "o": 128, "gate_up": B, "down": 128}),  # gate|up: 256 x 128 measured 194 us, 256 x 256 202
    ("1.7b", 4080, {"qkv": B, "o": 128, "gate_up": B, "down": 128}),
])
def test_prompt_gemm_tiles_at_the_benchmark_shapes(name, tokens, want):
    for g, (rows, k, epi) in _gemms(name).items():
        p = nnc.plan_prefill_gemm(rows, k, tokens, 1, epi)
        got = (p.tile_rows, p.tile_cols)
        assert got == (want[g] if isinstance(want[g], tuple) else (want[g], 128)), (g, got)
        assert p.k_slices == 1                                       # (no slices allowed in this call)
        assert p.t_us >= max(p.t_comp_us, p.t_mem_us)                # objective: max(T_mem, T_comp) + epilogue + launch


def test_model_times_are_close_to_the_measured_ones():
    # 8B shapes, 4080-token block, microseconds measured with HIP events around each launch
    measured = {"qkv": 164, "o": 126, "gate_up": 595, "down": 291}
    for g, (rows, k, epi) in _gemms("8b").items():
        p = nnc.plan_prefill_gemm(rows, k, 4080, 1, epi)
        assert abs(p.t_us - measured[g]) / measured[g] < 0.12, (g, p.t_us)
    # batched decode GEMMs of the 8B shape, 16 sequences x 3 pieces
    H, Dq, Dkv, F = SHAPES["8b"]
    # launches back to back of the kernel alone, 16 sequences x 3 pieces, at the model's pick
    for rows, k, epi, ks, us in ((Dq + 2 * Dkv, H, STORE, 1, 15.3), (Dq + 2 * Dkv, H, STORE, 4, 12.6), (H, Dq, STORE, 8, 9.9),
                                 (2 * F, H, SWIGLU, 1, 36.4), (H, F, STORE, 8, 21.7), (V, H, STORE, 1, 226.6)):
        p = nnc.plan_skinny_gemm(rows, k, 16, 3, epi, ks)
        assert abs(p.t_us - us) / us < 0.20, (rows, p.t_us)


def test_mid_size_blocks_split_k_of_the_residual_projections():
    """Blocks of 768 .. 2048 tokens give the O / down projections fewer 256- or 128-row tiles than the
    chip has CUs; the model then splits k on the direct-copy tiles too.  Measured per layer (O + down +
    the two norm kernels that add the partials, HIP events): 8B shape, 1024 tokens: 224 us unsliced at
    best, 192 at the pick below; 4B shape, 768 tokens: 181 -> 108; 4B, 2032: 212 -> 201; 8B, 2048:
    316 -> 290.  From 3072 tokens on the partials no longer stay in the caches and slicing loses."""
    H8, Dq8, _, F8 = SHAPES["8b"]
    H4, Dq4, _, F4 = SHAPES["4b"]
    RESID = 1
    for rows, k, tokens, tile, ks in ((H8, F8, 1024, (128, 128), 2), (H8, Dq8, 1024, (128, 128), 2),
                                      (H4, F4, 768, (128, 128), 4), (H4, F4, 2032, (192, 256), 2),
                                      (H8, F8, 2048, (256, 256), 2)):
        p = nnc.plan_prefill_gemm(rows, k, tokens, 1, RESID, 4)
        assert ((p.tile_rows, p.tile_cols), p.k_slices) == (tile, ks), (rows, k, tokens, p.tile_rows, p.tile_cols, p.k_slices)
        assert p.t_us < nnc.plan_prefill_gemm(rows, k, tokens, 1, RESID, 1).t_us
        assert (k // 32) / p.k_slices >= 16            # a slice keeps the three LDS stages busy
    for rows, k in ((H8, F8), (H8, Dq8), (H4, F4), (H4, Dq4)):
        assert nnc.plan_prefill_gemm(rows, k, 4080, 1, RESID, 4).k_slices == 1
    # only the residual projections have a consumer that adds partial sums
    assert nnc.plan_prefill_gemm(2 * F8, H8, 1024, 1, SWIGLU, 4).k_slices == 1


def test_short_prompts_are_memory_bound_and_may_split_k():
    # 128 tokens of the 0.6B shape: the narrow projections have too few tiles for the chip, the
    # model splits k (the epilogue adds partial sums) and picks small tiles
    rows, k, epi = _gemms("0.6b")["o"]
    one = nnc.plan_prefill_gemm(rows, k, 128, 2, epi, 1)
    many = nnc.plan_prefill_gemm(rows, k, 128, 2, epi, 4)
    assert many.k_slices > 1 and many.tile_rows == 64 and many.t_us < one.t_us
    assert many.workgroups >= 256
    # never beyond what the caller allows, never slices shorter than 8 k steps
    for ks in (1, 2, 3, 4):
        p = nnc.plan_prefill_gemm(rows, k, 128, 2, epi, ks)
        assert 1 <= p.k_slices <= ks and (k // 32) / p.k_slices >= 8
    # QKV cannot split (its consumer wants the full sums)
    rows, k, epi = _gemms("0.6b")["qkv"]
    assert nnc.plan_prefill_gemm(rows, k, 128, 2, epi, 1).k_slices == 1


def test_skinny_gemm_plans_at_the_batched_workloads():
    H, Dq, Dkv, F = SHAPES["8b"]
    # what a CU pulls through its vector memory path (weights + the operand of every workgroup it
    # runs) decides: one workgroup per CU with as many row tiles as that allows
    qkv = nnc.plan_skinny_gemm(Dq + 2 * Dkv, H, 16, 3, STORE)
    assert (qkv.tile_code, qkv.k_slices, qkv.workgroups) == (2, 1, 192)                 # no k split: 384 tiles as 192 x 2
    qkv = nnc.plan_skinny_gemm(Dq + 2 * Dkv, H, 16, 3, STORE, 4)
    assert (qkv.tile_code, qkv.k_slices, qkv.workgroups) == (3, 2, 256)                 # the consumer adds two k halves
    gu = nnc.plan_skinny_gemm(2 * F, H, 16, 3, SWIGLU)
    assert (gu.tile_code, gu.workgroups) == (6, 256)                                     # three (gate, up) pairs per CU
    o = nnc.plan_skinny_gemm(H, Dq, 16, 3, STORE, 8)
    assert (o.tile_code, o.k_slices, o.workgroups) == (2, 2, 256)
    head = nnc.plan_skinny_gemm(V, H, 16, 3, STORE)
    assert head.tile_code == 4                                                           # 9496 tiles: 1, 2 or 4 divide
    down = nnc.plan_skinny_gemm(H, F, 16, 3, STORE, 8)
    assert down.workgroups % 256 == 0 and 1 < down.k_slices <= 8
    # batch 1: nothing to re-read, the choice is about filling the chip
    assert nnc.plan_skinny_gemm(V, 1024, 1, 3, STORE).workgroups >= 2048
    H4, Dq4, _, F4 = SHAPES["4b"]
    d4 = nnc.plan_skinny_gemm(H4, F4, 8, 3, STORE, 8)
    assert (d4.tile_code, d4.k_slices, d4.workgroups) == (2, 3, 240)                     # 80 tile pairs x 3 slices
    g4 = nnc.plan_skinny_gemm(2 * F4, H4, 8, 3, SWIGLU)
    assert (g4.tile_code, g4.workgroups) == (2, 608)                                     # 152 workgroups of 8 tiles would leave 104 CUs idle


def test_planner_rejects_bad_shapes():
    with pytest.raises(nnc.NncError):
        nnc.plan_prefill_gemm(100, 4096, 128, 1, STORE)        # rows not a multiple of 16
    with pytest.raises(nnc.NncError):
        nnc.plan_skinny_gemm(4096, 4096, 30, 3, STORE)         # 90 operand columns: more than a pass carries
    with pytest.raises(nnc.NncError):
        nnc.plan_skinny_gemm(4096, 4096, 4, 3, RESID)          # no such epilogue for the streaming GEMM
