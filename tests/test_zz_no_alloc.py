"""The entry point that allocates nothing (moc_route_static, for callers that cannot call hipMalloc)
against moc_route, through the C ABI: pooled keys and selections must be identical bit for bit
(integer output: exact; the pooled means are the same kernel on the same inputs), on two calls in
a row, the second with a smaller input, so that what the first call left in the static scratch
array is seen not to leak into the second."""
import numpy as np
import pytest
import torch

import moc_inputs as mi
from paper_2508_21058_amd import binding as mb

pytestmark = pytest.mark.gpu


def _both(lay, B, H, d, topk, seed, dtype=torch.bfloat16, causal=True):
    q, k, _, _ = mi.qkv_do(B, H, lay.N, d, seed, "cuda")
    q, k = q.to(dtype).contiguous(), k.to(dtype).contiguous()
    meta = mb.chunk_meta(lay.offsets, lay.shot, lay.window, lay.text_spans)
    pooled_ref, sel_ref = mb.route(meta, q, k, topk, causal)
    pooled = torch.full_like(pooled_ref, float("nan"))
    sel = torch.full_like(sel_ref, -5)
    torch.cuda.synchronize()
    # torch's count of allocation requests so far: it only grows, so a tensor of an earlier test that
    # the garbage collector frees meanwhile does not disturb the comparison
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    mb.route_static(meta, q, k, topk, causal, out=(pooled, sel))
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before, "route_static allocated through torch"
    assert torch.equal(pooled, pooled_ref), "pooled keys differ"
    assert torch.equal(sel, sel_ref), "selections differ"
    meta.close()


def test_static_scratch_route_equals_route_twice_second_call_smaller():
    big = mi.multishot_layout(3, 40, 4, 520, 130, "frame")          # 51 chunks -> planes of 64 rows
    _both(big, 1, 4, 128, 5, seed=3)
    small = mi.multishot_layout(1, 16, 2, 96, 32, "chunk")          # 7 chunks -> planes of 32 rows
    _both(small, 1, 2, 128, 3, seed=4)
    _both(small, 2, 1, 64, 2, seed=5, dtype=torch.float32, causal=False)


def test_static_scratch_limit_is_enforced():
    """Shapes whose planes exceed MOC_STATIC_SCRATCH_BYTES (16 MiB) are refused before any launch."""
    C = 4096
    lay_off = np.arange(C + 1, dtype=np.int32) * 2
    meta = mb.chunk_meta(lay_off, np.zeros(C, np.int32), None, None)
    q = torch.zeros(1, 8, int(lay_off[-1]), 128, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(mb.MocError) as e:                              # 8 * 3 * 4096 * 128 * 2 = 24 MiB
        mb.route_static(meta, q, q, 2)
    assert e.value.status == -7
    mb.route_static(meta, q[:, :4].contiguous(), q[:, :4].contiguous(), 2)      # 12 MiB fits
    torch.cuda.synchronize()
    meta.close()
