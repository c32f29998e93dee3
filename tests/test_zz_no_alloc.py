"""prune_enumerate_static (the entry point that allocates nothing: its scratch is a fixed array in the
library's device data) against prune_enumerate, through the C ABI, to the same bar as the oracle tests:
integer outputs bit-exact, losses bit-identical (same kernels, same order)."""
import ctypes

import pytest
import torch

import paper_2402_14800_amd as pkg
from paper_2402_14800_amd import binding
from paper_2402_14800_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(logits, Y, k, r):
    ref = pkg.prune_enumerate(logits, Y, k, r)
    torch.cuda.synchronize()
    E = Y.shape[0]
    n = pkg.num_subsets(E, r)
    # outputs allocated up front and poisoned: the call itself must allocate nothing and overwrite them all
    out = (torch.full((n,), float("nan"), dtype=torch.float32, device=DEV),
           torch.full((1,), -7, dtype=torch.int32, device=DEV), torch.full((1,), -7, dtype=torch.int32, device=DEV),
           torch.full((1,), -7, dtype=torch.int64, device=DEV))
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats(DEV)["allocation.all.allocated"]
    got = pkg.prune_enumerate_static(logits, Y, k, r, out=out)
    after = torch.cuda.memory_stats(DEV)["allocation.all.allocated"]
    torch.cuda.synchronize()
    assert after == before                                   # torch's allocator was not asked for anything
    assert torch.equal(got[0].view(torch.int32), ref[0].view(torch.int32))
    assert torch.equal(got[1], ref[1]) and torch.equal(got[2], ref[2]) and torch.equal(got[3], ref[3])
    return ref


def test_static_scratch_entry_point_matches_prune_enumerate_twice_in_a_row():
    # first call: E = 8, r = 4 on 3000 tokens; second call right after it on a SMALLER input with another E, r and
    # dtype, so that every region of the shared scratch array holds the first call's leftovers
    logits1, Y1 = wl.make_enumeration_inputs(8, 3000, 256, "bf16", seed=71, device=DEV)
    ref1 = _both(logits1, Y1, 2, 4)
    logits2, Y2 = wl.make_enumeration_inputs(6, 517, 64, "f32", seed=72, device=DEV)
    _both(logits2, Y2, 2, 3)
    logits3, Y3 = wl.make_enumeration_inputs(16, 300, 128, "bf16", seed=73, bias_var=0.5, device=DEV)
    _both(logits3, Y3, 4, 12)
    # and the first input again: same bits as before
    again = pkg.prune_enumerate_static(logits1, Y1, 2, 4)
    torch.cuda.synchronize()
    assert torch.equal(again[0].view(torch.int32), ref1[0].view(torch.int32)) and torch.equal(again[1], ref1[1])


def test_static_scratch_entry_point_rejects_sizes_beyond_its_array():
    T, E, H, k, r = 200000, 8, 64, 2, 4
    assert binding.prune_enumerate_workspace(T, E, H, k, r, binding.MOEP_BF16) > binding.STATIC_SCRATCH_BYTES
    p = ctypes.c_void_p
    st = binding._lib.prune_enumerate_static(p(1 << 20), p(1 << 20), T, E, H, binding.MOEP_BF16, k, r,
                                             p(1 << 20), p(1 << 20), p(1 << 20), None, None)
    assert st == 3 and b"scratch" in binding._lib.moep_last_error()
    # an empty batch needs no scratch and gives zeros
    logits, Y = wl.make_enumeration_inputs(8, 16, 64, "bf16", seed=74, device=DEV)
    loss, amin, amask, unaff = pkg.prune_enumerate_static(logits[:0].contiguous(), Y[:, :0].contiguous(), 2, 6)
    torch.cuda.synchronize()
    assert loss.tolist() == [0.0] * 28 and amin.item() == 0 and unaff.item() == 0
