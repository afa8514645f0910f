"""The allocation-free entry point against the entry point it is a variant of: same kernels, scratch
memory in the library's own per-GPU array instead of a caller's workspace.  Two calls in a row, the
second on a smaller input (the array keeps the first call's contents)."""
import numpy as np
import pytest
import torch

import paper_1412_4526_amd as dsk

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(shape, frac, seed):
    N, Cls, H, W = shape
    rng = np.random.default_rng(seed)
    scores = torch.from_numpy((rng.standard_normal(shape) * 3).astype(np.float32)).to(DEV)
    labels = torch.from_numpy(rng.integers(0, Cls, (N, H, W)).astype(np.int32)).to(DEV)
    mask = torch.from_numpy((rng.random((N, H, W)) < frac).astype(np.uint8)).to(DEV)
    return scores, labels, mask


def test_static_scratch_entry_point_matches_the_workspace_one():
    for shape, frac, dt in (((2, 33, 300, 317), 0.05, torch.float32),      # several hundred workgroups
                            ((1, 10, 37, 41), 0.5, torch.float32),          # smaller, right after the larger one
                            ((1, 2, 64, 50), 1.0, torch.bfloat16),
                            ((1, 70, 20, 9), 0.0, torch.float32)):          # empty mask; more classes than registers hold
        print("static softmax", shape, frac, dt, flush=True)
        scores, labels, mask = _case(shape, frac, seed=shape[1])
        loss_ref, d_ref = dsk.dsk_masked_softmax_xent(scores, labels, mask, dscores_dtype=dt)
        loss = torch.full((1,), -7.0, device=DEV)
        d = torch.full(shape, 3.0, dtype=dt, device=DEV)
        before = torch.cuda.memory_allocated()
        dsk.dsk_masked_softmax_xent_static(scores, labels, mask, loss, d)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        assert torch.equal(loss, loss_ref), (loss.item(), loss_ref.item())
        assert torch.equal(d, d_ref)


def test_static_scratch_entry_point_rejects_what_it_cannot_hold():
    P = 0x1000
    L = dsk.lib
    assert L.dsk_masked_softmax_xent_static(P, P, P, P, P, 0, 64, 64, 1024, 1024, None) == dsk.DSK_ESHAPE   # 2^32 entries
    assert L.dsk_masked_softmax_xent_static(P, P, None, P, P, 0, 1, 5, 8, 8, None) == dsk.DSK_EINVAL
    assert L.dsk_masked_softmax_xent_static(P, P, P, P, P, 3, 1, 5, 8, 8, None) == dsk.DSK_EINVAL
