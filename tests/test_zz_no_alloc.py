"""GPU: the allocation-free selection (topk_by_loss_static) against topk_by_loss through the C ABI, bit for bit,
on calls in a row that share the library's fixed device array (the later ones on smaller pools)."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2508_08540_amd as bls
    ctx = bls.Context(0)
    yield torch, bls, ctx
    ctx.close()


def _both(torch, bls, ctx, arr, k):
    d = torch.from_numpy(arr).cuda()
    out = []
    for fn in (bls.topk_by_loss, bls.topk_by_loss_static):
        idx = torch.full((max(k, 1),), -1, dtype=torch.int32, device="cuda")
        val = torch.full((max(k, 1),), -7.0, dtype=torch.float32, device="cuda")
        fn(ctx, d, k, idx, val)
        ctx.synchronize()
        out.append((idx.cpu().numpy()[:k], val.cpu().numpy()[:k].view(np.uint32)))
    np.testing.assert_array_equal(out[1][0], out[0][0])
    np.testing.assert_array_equal(out[1][1], out[0][1])


def test_static_selection_equals_the_allocating_one_on_successive_calls():
    import torch
    import paper_2508_08540_amd as bls
    ctx = bls.Context(0)
    try:
        # large pool first, then smaller ones: the array keeps the earlier call's contents
        for kind, n in (("halfnormal", (1 << 20) - 5), ("ties16", 300000), ("specials", 70001), ("ties16", 16385), ("halfnormal", 4097),
                        ("specials", 100000)):
            arr = synth.loss_array(kind, n, seed=n)
            for k in (n // 4, 1, n):
                _both(torch, bls, ctx, arr, k)
        # the limit is enforced, and nothing is written
        big = torch.zeros(bls.TOPK_STATIC_MAX_N + 1, dtype=torch.float32, device="cuda")
        idx = torch.full((4,), -1, dtype=torch.int32, device="cuda")
        with pytest.raises(bls.BlsError):
            bls.topk_by_loss_static(ctx, big, 4, idx)
        ctx.synchronize()
        assert (idx.cpu().numpy() == -1).all()
        bls.topk_by_loss_static(ctx, big[:bls.TOPK_STATIC_MAX_N], 4, idx)   # at the limit: all equal, lowest indices
        ctx.synchronize()
        np.testing.assert_array_equal(idx.cpu().numpy(), np.arange(4))
    finally:
        ctx.close()


def test_static_selection_allocates_no_device_memory():
    import torch
    import paper_2508_08540_amd as bls
    ctx = bls.Context(0)
    try:
        arr = torch.from_numpy(synth.loss_array("halfnormal", 500000, seed=3)).cuda()
        idx = torch.empty(125000, dtype=torch.int32, device="cuda")
        bls.topk_by_loss_static(ctx, arr[:20000], 100, idx)      # first launches load the kernels
        ctx.synchronize()
        torch.cuda.synchronize()
        free0, _ = torch.cuda.mem_get_info()
        bls.topk_by_loss_static(ctx, arr, 125000, idx)
        ctx.synchronize()
        free1, _ = torch.cuda.mem_get_info()
        assert free1 == free0      # a fresh context has no scratch arena: the allocating call would have grown one here
    finally:
        ctx.close()
