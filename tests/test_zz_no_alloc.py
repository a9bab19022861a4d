"""GPU test of hdt_attn_bwd_no_alloc (the backward pass for callers that cannot allocate device memory) against
hdt_attn_bwd: same kernels, the workspace being the library's own array instead of the caller's, so the results
must be identical bit for bit.  Two calls in a row, the second on a smaller input: the array keeps the first
call's contents and nothing of them may show."""
import ctypes

import numpy as np
import pytest

from paper_2407_08330_amd import inputs
from gpu_common import make_inputs, say, to_dev_i32

pytestmark = pytest.mark.gpu


def both_ways(hdt, level, parent, H, D, seed, tile=(0, 0)):
    import torch
    B, N = level.shape
    scale = 1.0 / np.sqrt(D)
    _, (q, k, v, d_o) = make_inputs(B, H, N, D, seed, "bf16", n_tensors=4)
    lay = hdt.hdt_build_layout(to_dev_i32(level), to_dev_i32(parent), tile_m=tile[0], tile_n=tile[1])
    o, lse = hdt.hdt_attn_fwd(lay, q, k, v, scale)
    want = hdt.hdt_attn_bwd(lay, q, k, v, o, lse, d_o, scale)
    got = tuple(torch.full_like(q, float("nan")) for _ in range(3))
    torch.cuda.synchronize()
    # the binding asks torch for nothing (its count of allocations ever made does not move; the bytes in use may
    # drop at any time when Python collects an earlier test's tensors)
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    hdt.hdt_attn_bwd_no_alloc(lay, q, k, v, o, lse, d_o, scale, *got)
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
    torch.cuda.synchronize()
    for name, g, w in zip(("dq", "dk", "dv"), got, want):
        assert torch.equal(g.view(torch.int16), w.view(torch.int16)), f"{name} differs from hdt_attn_bwd"
    return lay


def test_no_alloc_backward_twice_the_second_call_smaller(oracle):
    import paper_2407_08330_amd as hdt
    big = inputs.make_workload(2, batch=2)
    say(f"[no-alloc] config 2 documents, B=2 H=4 N={big.n_pos} d=64")
    both_ways(hdt, big.level, big.parent, 4, 64, 31).destroy()
    small = inputs.make_workload(1)
    say(f"[no-alloc] config 1 document, B=1 H=2 N={small.n_pos} d=128, tile 64x32")
    both_ways(hdt, small.level, small.parent, 2, 128, 32, tile=(64, 32)).destroy()


def test_no_alloc_backward_refuses_what_does_not_fit():
    import torch
    import paper_2407_08330_amd as hdt
    # two floats of workspace per (batch, head, position): 2^20 + 2048 of them do not fit the 8 MiB array
    n, heads = 2048, 513
    level = np.full((1, n), 1, np.int32)
    level[0, 0] = 0
    parent = np.zeros((1, n), np.int32)
    parent[0, 0] = -1
    lay = hdt.hdt_build_layout(to_dev_i32(level), to_dev_i32(parent))
    assert hdt.hdt_attn_bwd_workspace_bytes(lay, heads, 64, 0) > (8 << 20)
    lib = hdt.load_library()
    x = torch.zeros(16, dtype=torch.bfloat16, device="cuda")   # never read: the size check comes first
    p = ctypes.c_void_p(x.data_ptr())
    st = lib.hdt_attn_bwd_no_alloc(lay.handle, p, p, p, p, p, p, p, p, p, heads, 64, 0, ctypes.c_float(0.125), None)
    assert lib.hdt_status_string(st).decode() == "HDT_ERR_SHAPE" and b"workspace" in lib.hdt_last_error()
    lay.destroy()
