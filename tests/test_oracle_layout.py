"""Pins for the oracle's key order and block schedule (App. A.1, Alg. 1: sort keys by level,
partition into blocks, skip blocks whose mask is all zero)."""
import numpy as np
import pytest

from paper_2407_08330_amd import inputs
from helpers import mask_from_equations, read_golden_mask


@pytest.mark.parametrize("name", ["mask_doc16.txt", "mask_tree10.txt"])
def test_kperm_hand_written(oracle, name):
    level, _, kperm, _ = read_golden_mask(name)
    np.testing.assert_array_equal(oracle.kperm(level), kperm)


def test_kperm_is_stable_sort_by_level(oracle):
    wl = inputs.make_workload(3, batch=1)
    level = wl.level[0]
    rank = np.where(level < 0, np.iinfo(np.int32).max, level)
    np.testing.assert_array_equal(oracle.kperm(level), np.argsort(rank, kind="stable"))


def _schedule_from_dense_mask(M, kperm, bm, bn):
    """Brute force in numpy from a dense mask pinned elsewhere."""
    n = M.shape[0]
    tr, tc = -(-n // bm), -(-n // bn)
    Mp = np.zeros((tr * bm, tc * bn), dtype=np.uint8)
    Mp[:n, :n] = M[:, kperm]
    blocks = Mp.reshape(tr, bm, tc, bn).transpose(0, 2, 1, 3)
    return blocks, blocks.reshape(tr, tc, -1).sum(axis=2)


@pytest.mark.parametrize("bm,bn", [(128, 64), (64, 32), (32, 32), (128, 128)])
def test_block_schedule_against_dense_mask(oracle, bm, bn):
    wl = inputs.make_workload(1)
    level, parent = wl.level[0], wl.parent[0]
    M = mask_from_equations(wl.sections[0], wl.n_pos)
    sch = oracle.block_schedule(level, parent, bm, bn)
    blocks, cnt = _schedule_from_dense_mask(M, sch.kperm, bm, bn)
    tr, tc = cnt.shape
    assert sch.nnz == M.sum()
    t = 0
    for I in range(tr):
        cols = np.nonzero(cnt[I])[0]
        np.testing.assert_array_equal(sch.q_cols[sch.q_rowptr[I]:sch.q_rowptr[I + 1]], cols)
        for J in cols:
            blk = blocks[I, J]
            assert sch.q_full[t] == (blk.all())
            # bitmap: word r*(bn/32)+c/32, bit c%32
            got = ((sch.bits[t][:, :, None] >> np.arange(32, dtype=np.uint32)) & 1).reshape(bm, bn)
            np.testing.assert_array_equal(got, blk)
            for r in range(bm // 32):
                for c in range(bn // 32):
                    sb = blk[r * 32:(r + 1) * 32, c * 32:(c + 1) * 32]
                    bit = r * (bn // 32) + c
                    assert ((sch.q_sub[t] >> bit) & 1) == sb.any()
                    assert ((sch.q_sub[t] >> (16 + bit)) & 1) == sb.all()
            t += 1
    assert t == sch.q_cols.shape[0]
    # transpose
    for J in range(tc):
        rows = np.nonzero(cnt[:, J])[0]
        np.testing.assert_array_equal(sch.k_rows[sch.k_colptr[J]:sch.k_colptr[J + 1]], rows)
        for e in range(sch.k_colptr[J], sch.k_colptr[J + 1]):
            tt = sch.k_tile[e]
            assert sch.q_cols[tt] == J
            assert sch.q_rowptr[sch.k_rows[e]] <= tt < sch.q_rowptr[sch.k_rows[e] + 1]


def test_ragged_length_and_hand_example(oracle):
    level, parent, kperm, M = read_golden_mask("mask_tree10.txt")   # n = 10, one ragged 32x32 block
    sch = oracle.block_schedule(level, parent, 32, 32)
    assert sch.q_rowptr.tolist() == [0, 1] and sch.q_cols.tolist() == [0] and sch.q_full.tolist() == [0]
    got = ((sch.bits[0][:, :, None] >> np.arange(32, dtype=np.uint32)) & 1).reshape(32, 32)
    np.testing.assert_array_equal(got[:10, :10], M[:, kperm])
    assert got[10:].sum() == 0 and got[:, 10:].sum() == 0
    assert sch.nnz == M.sum()


def test_every_allowed_pair_is_covered_and_no_block_is_empty(oracle):
    wl = inputs.make_workload(2, batch=1)
    level, parent = wl.level[0], wl.parent[0]
    sch = oracle.block_schedule(level, parent, 128, 64)
    rowptr, cols = oracle.row_lists(level, parent)
    slot = np.empty(wl.n_pos, dtype=np.int64)
    slot[sch.kperm] = np.arange(wl.n_pos)
    alive = set()
    for I in range(len(sch.q_rowptr) - 1):
        for J in sch.q_cols[sch.q_rowptr[I]:sch.q_rowptr[I + 1]]:
            alive.add((I, int(J)))
    rows = np.repeat(np.arange(wl.n_pos), np.diff(rowptr))
    needed = set(zip((rows // 128).tolist(), (slot[cols] // 64).tolist()))
    assert needed == alive
    assert all(b.any() for b in sch.bits)
    assert sch.nnz == rowptr[-1]


def test_sorting_keys_by_level_reduces_blocks(oracle):
    # the paper's claim behind the sort (Sec. 3.2; Fig. 6 caption)
    for cfg in (2, 3):
        wl = inputs.make_workload(cfg, batch=2)
        for s in range(2):
            a = oracle.block_schedule(wl.level[s], wl.parent[s], 128, 64, use_sort=True)
            b = oracle.block_schedule(wl.level[s], wl.parent[s], 128, 64, use_sort=False)
            assert a.q_cols.shape[0] < b.q_cols.shape[0]
            assert a.nnz == b.nnz


def test_force_dense_issues_every_block(oracle):
    wl = inputs.make_workload(1)
    sch = oracle.block_schedule(wl.level[0], wl.parent[0], 128, 64, force_dense=True)
    assert sch.q_cols.shape[0] == (512 // 128) * (512 // 64)
    assert sch.q_rowptr.tolist() == [0, 8, 16, 24, 32]


# ---- per-query-block key lists (the library's default schedule) ---------------------------------

def _read_golden_keylists(name):
    import os
    from helpers import GOLDEN
    bm = bn = None
    rowptr, keys, rows = None, [], []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            tok = line.split()
            if tok[0] == "bm":
                bm = int(tok[1])
            elif tok[0] == "bn":
                bn = int(tok[1])
            elif tok[0] == "rowptr":
                rowptr = [int(t) for t in tok[1:]]
            elif tok[0] == "entry":
                keys.append([int(t) for t in tok[1:]])
                rows.append([])
            else:
                rows[-1].append([int(c) for c in line])
    return bm, bn, np.array(rowptr), np.array(keys, np.int32), np.array(rows, np.uint8)


def _unpack(bits, bn):
    """uint32 [E][bm][wpr] -> 0/1 [E][bm][bn]"""
    b = (bits[:, :, :, None] >> np.arange(32, dtype=np.uint32)) & 1
    return b.reshape(bits.shape[0], bits.shape[1], -1)[:, :, :bn].astype(np.uint8)


def test_keylists_hand_written(oracle):
    level, parent, _, _ = read_golden_mask("mask_doc16.txt")
    bm, bn, rowptr, keys, rows = _read_golden_keylists("keylists_doc16.txt")
    sch = oracle.keylist_schedule(level, parent, bm, bn)
    np.testing.assert_array_equal(sch.q_rowptr, rowptr)
    np.testing.assert_array_equal(sch.q_keys, keys)
    np.testing.assert_array_equal(_unpack(sch.bits, bn), rows)
    np.testing.assert_array_equal(sch.pairs, rows.reshape(rows.shape[0], -1).sum(axis=1))


def _check_keylists_against_dense_mask(sch, M, kperm, bm, bn):
    """Everything the definition fixes, derived from a dense mask that is pinned elsewhere:
    the lists hold exactly the non-empty key columns of each query block, in key order, packed
    without gaps, and the bitmaps put back together give the mask."""
    n = M.shape[0]
    tr = -(-n // bm)
    slot = np.empty(n, dtype=np.int64)
    slot[kperm] = np.arange(n)
    rebuilt = np.zeros_like(M)
    dense_bits = _unpack(sch.bits, bn)
    assert sch.q_rowptr[0] == 0 and len(sch.q_rowptr) == tr + 1
    for I in range(tr):
        blk = M[I * bm:(I + 1) * bm]
        want = kperm[np.nonzero(blk[:, kperm].any(axis=0))[0]]      # non-empty columns, key order
        e0, e1 = sch.q_rowptr[I], sch.q_rowptr[I + 1]
        assert e1 - e0 == -(-len(want) // bn)
        flat = sch.q_keys[e0:e1].reshape(-1)
        np.testing.assert_array_equal(flat[:len(want)], want)
        assert (flat[len(want):] == -1).all()
        assert (np.diff(slot[flat[:len(want)]]) > 0).all()
        for e in range(e0, e1):
            for c in range(bn):
                j = sch.q_keys[e, c]
                col = dense_bits[e, :, c]
                if j < 0:
                    assert col.sum() == 0
                else:
                    assert rebuilt[I * bm:(I + 1) * bm, j].sum() == 0     # a key appears once per block
                    rebuilt[I * bm:(I + 1) * bm, j] = col[:blk.shape[0]]
                    assert col[blk.shape[0]:].sum() == 0                   # rows past n
                    assert col.sum() > 0
    np.testing.assert_array_equal(rebuilt, M)
    assert sch.nnz == M.sum()
    np.testing.assert_array_equal(sch.pairs, dense_bits.reshape(dense_bits.shape[0], -1).sum(axis=1))


@pytest.mark.parametrize("bm,bn", [(128, 64), (32, 32), (64, 96), (128, 128)])
def test_keylists_against_equation_mask(oracle, bm, bn):
    wl = inputs.make_workload(1)
    M = mask_from_equations(wl.sections[0], wl.n_pos)
    level = wl.level[0]
    kp = np.argsort(np.where(level < 0, np.iinfo(np.int32).max, level), kind="stable")
    sch = oracle.keylist_schedule(level, wl.parent[0], bm, bn)
    _check_keylists_against_dense_mask(sch, M, kp, bm, bn)
    # sub-block summaries from the unpacked bitmaps
    d = _unpack(sch.bits, bn)
    for e in range(d.shape[0]):
        for r in range(bm // 32):
            for c in range(bn // 32):
                sb = d[e, r * 32:(r + 1) * 32, c * 32:(c + 1) * 32]
                bit = r * (bn // 32) + c
                assert ((sch.q_sub[e] >> bit) & 1) == sb.any()
                assert ((sch.q_sub[e] >> (16 + bit)) & 1) == sb.all()


@pytest.mark.parametrize("name", ["mask_doc16.txt", "mask_tree10.txt"])
def test_keylists_against_hand_masks(oracle, name):
    level, parent, kperm, M = read_golden_mask(name)
    for bm, bn in [(4, 4), (3, 5), (32, 32)]:
        sch = oracle.keylist_schedule(level, parent, bm, bn)
        _check_keylists_against_dense_mask(sch, M, kperm, bm, bn)


def test_keylists_without_sort_list_keys_in_document_order(oracle):
    level, parent, _, M = read_golden_mask("mask_doc16.txt")
    sch = oracle.keylist_schedule(level, parent, 4, 4, use_sort=False)
    _check_keylists_against_dense_mask(sch, M, np.arange(16), 4, 4)


def test_keylists_need_fewer_entries_than_windows(oracle):
    # the point of the refinement: fewer gathered key tiles for the same mask
    for cfg in (2, 3):
        wl = inputs.make_workload(cfg, batch=1)
        a = oracle.keylist_schedule(wl.level[0], wl.parent[0], 128, 64)
        b = oracle.block_schedule(wl.level[0], wl.parent[0], 128, 64)
        assert a.q_keys.shape[0] < 0.75 * b.q_cols.shape[0]
        assert a.nnz == b.nnz


def test_window_schedule_key_positions(oracle):
    # positions behind the key slots of the windowed schedule: kperm cut into windows, pads -> -1
    level, parent, kperm, _ = read_golden_mask("mask_doc16.txt")
    level = np.concatenate([level, np.full(48, -1, np.int32)])
    parent = np.concatenate([parent, np.full(48, -1, np.int32)])
    sch = oracle.block_schedule(level, parent, 32, 32)
    assert sch.q_cols.tolist() == [0]
    assert sch.q_keys[0].tolist() == kperm[:12].tolist() + [-1] * 20


@pytest.mark.parametrize("variant,kinds", [("gb", 2 | 4), ("blue", 4)])
def test_schedules_of_the_listops_variants(oracle, variant, kinds):
    # asymmetric masks (Sec. 4.1): the schedules describe the thinned mask, rows = queries
    import test_oracle_mask
    level, parent, kperm, _ = read_golden_mask("mask_tree10.txt")
    M = test_oracle_mask._read_variants("mask_tree10_variants.txt")[variant]
    with oracle.edges(kinds):
        for bm, bn in [(4, 4), (32, 32)]:
            _check_keylists_against_dense_mask(oracle.keylist_schedule(level, parent, bm, bn), M, kperm, bm, bn)
        sch = oracle.block_schedule(level, parent, 32, 32)
    got = ((sch.bits[0][:, :, None] >> np.arange(32, dtype=np.uint32)) & 1).reshape(32, 32)
    np.testing.assert_array_equal(got[:10, :10], M[:, kperm])
    assert sch.nnz == M.sum()
