"""Helpers for the GPU parity tests: move seeded inputs to the device, call the C ABI through the
binding, bring results back as numpy."""
import sys

import numpy as np

from paper_2407_08330_amd import inputs


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def to_dev_i32(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def to_dev_bf16(x32):
    """float32 numpy values that are already bf16-representable -> bf16 device tensor."""
    import torch
    bits = inputs.bf16_bits(x32)
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def from_dev(t):
    """device tensor (bf16 or fp32) -> float32 numpy"""
    import torch
    if t.dtype == torch.bfloat16:
        bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return inputs.bf16_bits_to_f32(bits)
    return t.float().cpu().numpy()


class GuardedWorkspace:
    """A device workspace of exactly `nbytes` bytes with a patterned guard behind it: `view` is what a call gets,
    `check()` says whether the call stayed inside it."""

    def __init__(self, nbytes, guard=4096):
        import torch
        self.nbytes = max(int(nbytes), 16)
        self.buf = torch.full((self.nbytes + guard,), 0x5A, dtype=torch.uint8, device="cuda")
        self.view = self.buf[:self.nbytes]

    def check(self):
        tail = self.buf[self.nbytes:]
        assert bool((tail == 0x5A).all()), "the call wrote behind the workspace it was given"


def make_inputs(B, H, N, D, seed, dtype, n_tensors=3):
    """Seeded N(0,1) tensors; for bf16 they are rounded first so that both sides see the same values."""
    xs = inputs.make_qkv(B, H, N, D, seed, n_tensors)
    if dtype == "bf16":
        xs = [inputs.round_to_bf16(x) for x in xs]
        dev = [to_dev_bf16(x) for x in xs]
    else:
        import torch
        dev = [torch.from_numpy(x).cuda() for x in xs]
    return xs, dev


def compare_layout(oracle, layout, level, parent, bm, bn, windowed=False, edges=0, **kw):
    """Bit-exact comparison of every exported array of every sample with the oracle's schedule:
    the per-query-tile key lists (default) or the windowed block schedule; ``edges`` selects the
    edge kinds both sides use."""
    with oracle.edges(edges or oracle.EDGE_ALL):
        return _compare_layout(oracle, layout, level, parent, bm, bn, windowed, **kw)


def _compare_layout(oracle, layout, level, parent, bm, bn, windowed=False, **kw):
    B = level.shape[0]
    total_tiles = total_nnz = 0
    assert bool(layout.info()["windowed"]) == bool(windowed or kw.get("force_dense"))
    for b in range(B):
        got = layout.export(b)
        if windowed or kw.get("force_dense"):
            ref = oracle.block_schedule(level[b], parent[b], bm, bn, **kw)
            np.testing.assert_array_equal(got["q_cols"], ref.q_cols, err_msg=f"q_cols sample {b}")
            np.testing.assert_array_equal(got["k_colptr"], ref.k_colptr, err_msg=f"k_colptr sample {b}")
            np.testing.assert_array_equal(got["k_rows"], ref.k_rows, err_msg=f"k_rows sample {b}")
            np.testing.assert_array_equal(got["k_tile"], ref.k_tile, err_msg=f"k_tile sample {b}")
        else:
            ref = oracle.keylist_schedule(level[b], parent[b], bm, bn, **kw)
            ordinal = np.arange(ref.q_keys.shape[0]) - np.repeat(ref.q_rowptr[:-1], np.diff(ref.q_rowptr))
            np.testing.assert_array_equal(got["q_cols"], ordinal, err_msg=f"entry ordinals sample {b}")
            assert "k_rows" not in got
        np.testing.assert_array_equal(got["kperm"], ref.kperm, err_msg=f"kperm sample {b}")
        np.testing.assert_array_equal(got["q_rowptr"], ref.q_rowptr, err_msg=f"q_rowptr sample {b}")
        exp_keys, exp_sub = ref.q_keys, ref.q_sub
        if windowed or kw.get("force_dense"):
            # a window keeps a key only where some row of the query tile may attend to it (the library gathers
            # nothing else); the dense baseline computes every sub-block of every tile
            cols = np.arange(bn)
            seen = np.bitwise_or.reduce(ref.bits.reshape(-1, bm, bn // 32), axis=1)
            seen = (seen[:, cols >> 5] >> (cols & 31).astype(np.uint32)) & 1
            exp_keys = np.where(seen.astype(bool), ref.q_keys.reshape(-1, bn), -1).reshape(ref.q_keys.shape)
            if kw.get("force_dense"):
                exp_sub = ref.q_sub | np.uint32((1 << ((bm // 32) * (bn // 32))) - 1)
        np.testing.assert_array_equal(got["q_keys"], exp_keys, err_msg=f"q_keys sample {b}")
        np.testing.assert_array_equal(got["q_sub"], exp_sub, err_msg=f"q_sub sample {b}")
        np.testing.assert_array_equal(got["bits"], ref.bits, err_msg=f"bits sample {b}")
        n_tiles, nnz = layout.sample_info(b)
        assert n_tiles == ref.q_keys.shape[0] and nnz == ref.nnz
        total_tiles += n_tiles
        total_nnz += nnz
    info = layout.info()
    assert info["n_tiles"] == total_tiles and info["nnz"] == total_nnz
    return total_tiles, total_nnz
