"""Pins of the cross-attention oracle (decoder rows attending to a level subset of the encoder's positions,
paper Sec. 4.2): subsets and schedules written out by hand, the textbook dense attention it must reduce to,
finite differences, and what must not depend on invisible positions."""
import os

import numpy as np
import pytest
import scipy.special

from helpers import read_golden_mask

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "cross_doc16.txt")


def _read_golden():
    masks, fwd, tr = {}, [], []
    for line in open(GOLDEN):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "mask":
            masks[int(t[1])] = [int(x) for x in t[2:]]
        else:
            rec = (int(t[1]), int(t[2]), [int(x) for x in t[3:7]], t[7], int(t[8]))
            (fwd if t[0] == "fwd" else tr).append(rec)
    return masks, fwd, tr


def test_visible_subsets_written_out_by_hand(oracle):
    level, _, _, _ = read_golden_mask("mask_doc16.txt")
    masks, _, _ = _read_golden()
    assert len(masks) == 7
    for m, want in masks.items():
        assert oracle.cross_select(level, m).tolist() == want, m


def _check_schedule(sch, want, n_blocks):
    got = []
    for I in range(n_blocks):
        for j, e in enumerate(range(sch.q_rowptr[I], sch.q_rowptr[I + 1])):
            rows = "".join("1" if sch.bits[e, r, 0] else "0" for r in range(sch.bm))
            # within a row every listed key is allowed: the row's word is the set of filled slots
            filled = sum(1 << c for c in range(sch.bn) if sch.q_keys[e, c] >= 0)
            assert all(int(sch.bits[e, r, 0]) in (0, filled) for r in range(sch.bm))
            got.append((I, j, sch.q_keys[e].tolist(), rows, int(sch.pairs[e])))
    assert got == want


def test_schedules_written_out_by_hand(oracle):
    level, _, _, _ = read_golden_mask("mask_doc16.txt")
    _, fwd, tr = _read_golden()
    f, t = oracle.cross_schedule(level, 6, 6, 4, 4)
    _check_schedule(f, fwd, 2)
    _check_schedule(t, tr, 4)
    assert f.nnz == t.nnz == 6 * 5


@pytest.mark.parametrize("level_mask", [2, 6, 14, 15])
def test_schedules_reproduce_the_dense_rectangle(oracle, level_mask):
    # both schedules, expanded entry by entry, give the same 0/1 matrix: row i, column j <=> j visible
    rng = np.random.default_rng(5)
    n_enc, n_dec, bm, bn = 200, 75, 32, 32
    level = rng.integers(-1, 4, size=n_enc).astype(np.int32)
    vis = np.array([l >= 0 and (level_mask >> l) & 1 for l in level], bool)
    want = np.broadcast_to(vis[None, :], (n_dec, n_enc))
    f, t = oracle.cross_schedule(level, n_dec, level_mask, bm, bn)
    got = np.zeros((n_dec, n_enc), bool)
    for I in range(len(f.q_rowptr) - 1):
        seen = []
        for e in range(f.q_rowptr[I], f.q_rowptr[I + 1]):
            for c in range(bn):
                j = f.q_keys[e, c]
                if j >= 0:
                    seen.append(j)
                for r in range(bm):
                    if (f.bits[e, r, c >> 5] >> (c & 31)) & 1:
                        assert j >= 0 and I * bm + r < n_dec
                        got[I * bm + r, j] = True
        assert seen == np.flatnonzero(vis).tolist()   # document order, nothing twice
    assert (got == want).all()
    got_t = np.zeros((n_dec, n_enc), bool)
    for I in range(len(t.q_rowptr) - 1):
        for e in range(t.q_rowptr[I], t.q_rowptr[I + 1]):
            for c in range(bn):
                i = t.q_keys[e, c]
                for r in range(bm):
                    if (t.bits[e, r, c >> 5] >> (c & 31)) & 1:
                        assert i >= 0 and I * bm + r < n_enc
                        assert not got_t[i, I * bm + r]
                        got_t[i, I * bm + r] = True
    assert (got_t == want).all()


def _inputs(rng, B, H, nd, ne, d):
    return [rng.standard_normal((B, H, n, d)) for n in (nd, ne, ne, nd)]


def test_all_positions_visible_is_textbook_dense_attention(oracle):
    rng = np.random.default_rng(1)
    B, H, nd, ne, d = 2, 3, 7, 11, 8
    q, k, v, _ = _inputs(rng, B, H, nd, ne, d)
    level = np.full((B, ne), 3, np.int32)
    scale = 0.37
    o, lse = oracle.cross_attn_fwd(q, k, v, level, 1 << 3, scale)
    s = scale * (q @ k.transpose(0, 1, 3, 2))
    assert np.allclose(o, scipy.special.softmax(s, axis=-1) @ v, atol=1e-12)
    assert np.allclose(lse, scipy.special.logsumexp(s, axis=-1), atol=1e-12)


def test_subset_is_dense_attention_on_the_gathered_rows(oracle):
    rng = np.random.default_rng(2)
    B, H, nd, ne, d = 2, 2, 5, 16, 4
    level, _, _, _ = read_golden_mask("mask_doc16.txt")
    level = np.stack([level, np.roll(level, 3)])
    q, k, v, d_o = _inputs(rng, B, H, nd, ne, d)
    for m in (2, 6, 14):
        o, lse = oracle.cross_attn_fwd(q, k, v, level, m, 0.5)
        dq, dk, dv = oracle.cross_attn_bwd(q, k, v, d_o, level, m, 0.5)
        for b in range(B):
            sel = [j for j in range(ne) if level[b, j] >= 0 and (m >> level[b, j]) & 1]
            s = 0.5 * (q[b] @ k[b][:, sel].transpose(0, 2, 1))
            assert np.allclose(o[b], scipy.special.softmax(s, axis=-1) @ v[b][:, sel], atol=1e-12)
            assert np.allclose(lse[b], scipy.special.logsumexp(s, axis=-1), atol=1e-12)
            hidden = [j for j in range(ne) if j not in sel]
            assert (dk[b][:, hidden] == 0).all() and (dv[b][:, hidden] == 0).all()
            # invisible rows do not matter: perturb them, nothing changes
            k2, v2 = k.copy(), v.copy()
            k2[b][:, hidden] += 10.0
            v2[b][:, hidden] -= 7.0
            o2, _ = oracle.cross_attn_fwd(q, k2, v2, level, m, 0.5)
            assert np.array_equal(o2[b], o[b])


def test_gradients_by_finite_differences(oracle):
    rng = np.random.default_rng(3)
    B, H, nd, ne, d = 1, 2, 4, 16, 3
    level, _, _, _ = read_golden_mask("mask_doc16.txt")
    level = level[None]
    q, k, v, d_o = _inputs(rng, B, H, nd, ne, d)
    m, scale, eps = 6, 0.8, 1e-6
    dq, dk, dv = oracle.cross_attn_bwd(q, k, v, d_o, level, m, scale)

    def loss(q_, k_, v_):
        return float((oracle.cross_attn_fwd(q_, k_, v_, level, m, scale)[0] * d_o).sum())

    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        for _ in range(25):
            idx = tuple(rng.integers(0, s) for s in x.shape)
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps
            xm[idx] -= eps
            args_p = {"q": (xp, k, v), "k": (q, xp, v), "v": (q, k, xp)}[name]
            args_m = {"q": (xm, k, v), "k": (q, xm, v), "v": (q, k, xm)}[name]
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(fd - g[idx]) < 1e-6 * max(1.0, abs(fd)), (name, idx)


def test_no_visible_position_gives_zero_and_minus_infinity(oracle):
    rng = np.random.default_rng(4)
    q, k, v, d_o = _inputs(rng, 1, 1, 3, 5, 2)
    level = np.full((1, 5), -1, np.int32)
    o, lse = oracle.cross_attn_fwd(q, k, v, level, 15, 1.0)
    assert (o == 0).all() and np.isneginf(lse).all()
    assert all((g == 0).all() for g in oracle.cross_attn_bwd(q, k, v, d_o, level, 15, 1.0))
