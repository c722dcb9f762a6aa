"""nnc_decode_step_static (the decode step that allocates nothing) against nnc_decode_step.

Two calls in a row on one model, the second with a smaller batch, each compared bit for bit
with the existing entry point on a second model that holds the same weights and the same
cache state.  Collected last on purpose (file name): a failure here must not hide other tests.
"""
import numpy as np
import pytest
import torch

import synth
from parity_util import SMALL_BF16, SMALL_G4

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nnc():
    from paper_2512_21571_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("shape", [SMALL_BF16, SMALL_G4], ids=lambda s: s.name)
def test_static_workspace_step_equals_decode_step_twice_in_a_row(nnc, shape):
    print(f"case: decode step without allocation, {shape.name}", flush=True)
    blob = synth.make_blob(shape, weight_std=0.05)
    B, ctx = 5, 200
    a = nnc.Model(shape, blob, B, ctx + 8)       # existing entry point
    b = nnc.Model(shape, blob, B, ctx + 8)       # entry point under test
    lens = [ctx, 3, 64, 65, 130]                # ragged contexts, chunk boundaries included
    firsts = []
    for s, n in enumerate(lens):
        toks = synth.tokens(n, shape.vocab, stream=s)
        _, na = a.prefill(s, toks)
        _, nb = b.prefill(s, toks)
        assert int(na.item()) == int(nb.item())
        firsts.append(int(na.item()))
    dev = a.device
    with torch.cuda.stream(b.stream):
        logits = torch.empty((B, shape.vocab), dtype=torch.float32, device=dev)
        nxt = torch.empty((B,), dtype=torch.int32, device=dev)
    # call 1: all five sequences
    slots = list(range(B))
    la, na = a.decode_step(slots, firsts)
    b.decode_step_static(slots, firsts, logits, nxt)
    torch.cuda.synchronize()
    assert torch.equal(la, logits) and torch.equal(na, nxt)
    t2 = [int(v) for v in na.tolist()]
    # call 2, right after, smaller: two of the sequences, in another order, no logits buffer
    sub = [3, 1]
    la2, na2 = a.decode_step(sub, [t2[3], t2[1]])
    nxt2 = torch.empty((2,), dtype=torch.int32, device=dev)
    b.decode_step_static(sub, [t2[3], t2[1]], None, nxt2)
    torch.cuda.synchronize()
    assert torch.equal(na2, nxt2)
    assert b.slot_len(3) == a.slot_len(3) == lens[3] + 2 and b.slot_len(0) == lens[0] + 1
    # and once more with logits, to see that the cache rows both calls appended are the same
    la3, na3 = a.decode_step(sub, [int(v) for v in na2.tolist()])
    lg3 = torch.empty((2, shape.vocab), dtype=torch.float32, device=dev)
    b.decode_step_static(sub, [int(v) for v in na2.tolist()], lg3, None)
    torch.cuda.synchronize()
    assert torch.equal(la3, lg3)
    assert np.isfinite(lg3.cpu().numpy()).all()


def test_static_workspace_limits_are_errors(nnc):
    shape = SMALL_BF16
    blob = synth.make_blob(shape, weight_std=0.05)
    m = nnc.Model(shape, blob, 12, 16)
    for s in range(12):
        m.prefill(s, synth.tokens(2, shape.vocab, stream=s), want_logits=False)
    with pytest.raises(nnc.NncError) as e:
        m.decode_step_static(list(range(9)), [1] * 9, None, None)     # more than NNC_STATIC_MAX_BATCH
    assert e.value.status == nnc.E_ARG and "static workspace" in str(e.value)
    assert m.slot_len(0) == 2                                           # state untouched
    m.profile_begin()
    with pytest.raises(nnc.NncError) as e:
        m.decode_step_static([0], [1], None, None)
    assert e.value.status == nnc.E_STATE
    m.profile_end()
