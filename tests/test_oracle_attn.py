"""Pins for the oracle's forward and backward: dense softmax attention as the special case of a
one-group document (paper Eq. 1), a textbook dense masked softmax on masks pinned elsewhere,
closed forms, and brute-force finite differences / an autograd of the dense definition."""
import numpy as np
import pytest
import torch

from paper_2407_08330_amd import inputs
from helpers import dense_masked_attention, mask_from_equations, read_golden_mask


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_one_group_document_is_dense_attention(oracle):
    # a root with n-1 children: everybody is parent, child or sibling of everybody -> all-ones mask
    n, d, H = 37, 8, 2
    level = np.array([0] + [1] * (n - 1), dtype=np.int32)
    parent = np.array([-1] + [0] * (n - 1), dtype=np.int32)
    assert oracle.mask(level, parent).all()
    q, k, v = (_rand((1, H, n, d), s) for s in (1, 2, 3))
    scale = 1.0 / np.sqrt(d)
    o, lse = oracle.attn_fwd(q, k, v, level[None], parent[None], scale)
    for h in range(H):
        a = scale * q[0, h] @ k[0, h].T                      # Eq. 1, no mask
        a = a - a.max(axis=1, keepdims=True)
        s = np.exp(a) / np.exp(a).sum(axis=1, keepdims=True)
        np.testing.assert_allclose(o[0, h], s @ v[0, h], rtol=1e-12, atol=1e-13)
        ref_lse = np.log(np.exp(scale * q[0, h] @ k[0, h].T).sum(axis=1))
        np.testing.assert_allclose(lse[0, h], ref_lse, rtol=1e-12, atol=1e-12)


def test_one_sentence_document_rows_are_dense_over_their_groups(oracle):
    # [DOC] [SEC] [SENT] t t t t t : token rows = dense attention over {SENT, tokens}
    level, parent = inputs.document_from_sections([[5]], 8)
    d = 4
    q, k, v = (_rand((1, 1, 8, d), s) for s in (4, 5, 6))
    o, lse = oracle.attn_fwd(q, k, v, level[None], parent[None], 0.5)
    groups = {0: [0, 1], 1: [0, 1, 2], 2: [1, 2, 3, 4, 5, 6, 7]}
    for t in range(3, 8):
        groups[t] = [2, 3, 4, 5, 6, 7]
    for i, g in groups.items():
        a = 0.5 * k[0, 0, g] @ q[0, 0, i]
        w = np.exp(a - a.max())
        w /= w.sum()
        np.testing.assert_allclose(o[0, 0, i], w @ v[0, 0, g], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(lse[0, 0, i], np.log(np.exp(a).sum()), rtol=1e-12)


@pytest.mark.parametrize("name", ["mask_doc16.txt", "mask_tree10.txt"])
def test_forward_against_textbook_masked_softmax_on_hand_masks(oracle, name):
    level, parent, _, M = read_golden_mask(name)
    n, d, H = level.shape[0], 6, 3
    q, k, v = (_rand((1, H, n, d), s) for s in (7, 8, 9))
    o, lse = oracle.attn_fwd(q, k, v, level[None], parent[None], 0.3)
    for h in range(H):
        o_ref, lse_ref, _ = dense_masked_attention(q[0, h], k[0, h], v[0, h], M, 0.3)
        np.testing.assert_allclose(o[0, h], o_ref, rtol=1e-12, atol=1e-13)
        np.testing.assert_array_equal(np.isneginf(lse[0, h]), np.isneginf(lse_ref))
        fin = np.isfinite(lse_ref)
        np.testing.assert_allclose(lse[0, h][fin], lse_ref[fin], rtol=1e-12)
        assert (o[0, h][~fin] == 0).all()        # pad rows: o = 0, lse = -inf


def test_forward_against_textbook_on_equation_mask_config1(oracle):
    wl = inputs.make_workload(1)
    M = mask_from_equations(wl.sections[0], wl.n_pos)
    d = 16
    q, k, v = (_rand((1, 2, wl.n_pos, d), s) for s in (10, 11, 12))
    o, lse = oracle.attn_fwd(q, k, v, wl.level, wl.parent, 0.25)
    for h in range(2):
        o_ref, lse_ref, _ = dense_masked_attention(q[0, h], k[0, h], v[0, h], M, 0.25)
        np.testing.assert_allclose(o[0, h], o_ref, rtol=1e-11, atol=1e-12)
        fin = np.isfinite(lse_ref)
        np.testing.assert_allclose(lse[0, h][fin], lse_ref[fin], rtol=1e-12)
        assert np.isneginf(lse[0, h][~fin]).all()


def test_forward_closed_forms(oracle):
    level, parent, _, M = read_golden_mask("mask_doc16.txt")
    n, d = 16, 5
    k, v = _rand((1, 1, n, d), 13), _rand((1, 1, n, d), 14)
    # Q = 0: uniform weights over the allowed keys
    o, lse = oracle.attn_fwd(np.zeros((1, 1, n, d)), k, v, level[None], parent[None], 1.0)
    cnt = M.sum(axis=1)
    for i in range(n):
        if cnt[i]:
            np.testing.assert_allclose(o[0, 0, i], v[0, 0, M[i].astype(bool)].mean(axis=0), rtol=1e-13, atol=1e-14)
            np.testing.assert_allclose(lse[0, 0, i], np.log(cnt[i]), rtol=1e-13)
    # V = const: O = const on every non-pad row
    q = _rand((1, 1, n, d), 15)
    o, _ = oracle.attn_fwd(q, k, np.full((1, 1, n, d), 2.5), level[None], parent[None], 0.7)
    np.testing.assert_allclose(o[0, 0, cnt > 0], 2.5, rtol=1e-13)
    # scale is applied to the logits: doubling scale == doubling q
    o1, l1 = oracle.attn_fwd(q, k, v, level[None], parent[None], 0.8)
    o2, l2 = oracle.attn_fwd(2 * q, k, v, level[None], parent[None], 0.4)
    np.testing.assert_allclose(o1, o2, rtol=1e-12, atol=1e-14)


def _loss(oracle, q, k, v, d_o, level, parent, scale):
    o, _ = oracle.attn_fwd(q, k, v, level, parent, scale)
    return float((o * d_o).sum())


@pytest.mark.parametrize("name", ["mask_doc16.txt", "mask_tree10.txt"])
def test_backward_finite_differences(oracle, name):
    level, parent, _, _ = read_golden_mask(name)
    n, d, H = level.shape[0], 3, 2
    q, k, v, d_o = (_rand((1, H, n, d), s) for s in (20, 21, 22, 23))
    lv, pr = level[None], parent[None]
    scale = 0.6
    dq, dk, dv = oracle.attn_bwd(q, k, v, d_o, lv, pr, scale)
    eps = 1e-6
    for name_, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = x[idx]
            x[idx] = old + eps
            lp = _loss(oracle, q, k, v, d_o, lv, pr, scale)
            x[idx] = old - eps
            lm = _loss(oracle, q, k, v, d_o, lv, pr, scale)
            x[idx] = old
            num[idx] = (lp - lm) / (2 * eps)
        np.testing.assert_allclose(g, num, rtol=2e-6, atol=2e-8, err_msg=name_)
    # gradients vanish on pads
    pads = level < 0
    assert (dq[0, :, pads] == 0).all() and (dk[0, :, pads] == 0).all() and (dv[0, :, pads] == 0).all()


def test_backward_against_autograd_of_dense_definition(oracle):
    wl = inputs.make_workload(1)
    n, d, H = 192, 8, 2
    level, parent = wl.level[:, :n], wl.parent[:, :n]
    M = torch.from_numpy(mask_from_equations(wl.sections[0], wl.n_pos)[:n, :n].astype(bool))
    q, k, v, d_o = (torch.from_numpy(_rand((1, H, n, d), s)).requires_grad_(s != 33) for s in (30, 31, 32, 33))
    scale = 1.0 / np.sqrt(d)
    a = scale * q @ k.transpose(-1, -2)
    a = a.masked_fill(~M, float("-inf"))
    s = torch.softmax(a, dim=-1)
    o = s @ v
    (o * d_o).sum().backward()
    dq, dk, dv = oracle.attn_bwd(q.detach().numpy(), k.detach().numpy(), v.detach().numpy(), d_o.numpy(),
                                 level, parent, scale)
    np.testing.assert_allclose(dq, q.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dk, k.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dv, v.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_backward_closed_form_q_zero(oracle):
    # Q = 0 => p_ij = 1/rowcount_i, so dV_j = sum_i allowed(i,j) dO_i / rowcount_i
    level, parent, _, M = read_golden_mask("mask_doc16.txt")
    n, d = 16, 4
    k, v, d_o = (_rand((1, 1, n, d), s) for s in (40, 41, 42))
    _, _, dv = oracle.attn_bwd(np.zeros((1, 1, n, d)), k, v, d_o, level[None], parent[None], 1.0)
    cnt = M.sum(axis=1).astype(np.float64)
    w = np.divide(M, cnt[:, None], out=np.zeros((n, n)), where=cnt[:, None] > 0)
    np.testing.assert_allclose(dv[0, 0], w.T @ d_o[0, 0], rtol=1e-12, atol=1e-14)


# ---- the thinned patterns of Sec. 4.1 (asymmetric masks) ------------------------------------------

def _variant_masks():
    import test_oracle_mask
    return test_oracle_mask._read_variants("mask_tree10_variants.txt")


@pytest.mark.parametrize("variant,kinds", [("gb", 2 | 4), ("blue", 4)])
def test_forward_on_listops_variants_against_textbook(oracle, variant, kinds):
    level, parent, _, _ = read_golden_mask("mask_tree10.txt")
    M = _variant_masks()[variant]
    n, d, H = level.shape[0], 5, 2
    q, k, v = (_rand((1, H, n, d), s) for s in (31, 32, 33))
    with oracle.edges(kinds):
        o, lse = oracle.attn_fwd(q, k, v, level[None], parent[None], 0.45)
    for h in range(H):
        o_ref, lse_ref, _ = dense_masked_attention(q[0, h], k[0, h], v[0, h], M, 0.45)
        np.testing.assert_allclose(o[0, h], o_ref, rtol=1e-12, atol=1e-13)
        fin = np.isfinite(lse_ref)
        np.testing.assert_allclose(lse[0, h][fin], lse_ref[fin], rtol=1e-12)
        assert np.isneginf(lse[0, h][~fin]).all()


@pytest.mark.parametrize("kinds", [2 | 4, 4, 1 | 2])
def test_backward_finite_differences_on_asymmetric_masks(oracle, kinds):
    level, parent, _, _ = read_golden_mask("mask_tree10.txt")
    n, d, H = level.shape[0], 3, 1
    q, k, v, d_o = (_rand((1, H, n, d), s) for s in (40, 41, 42, 43))
    lv, pr = level[None], parent[None]
    with oracle.edges(kinds):
        dq, dk, dv = oracle.attn_bwd(q, k, v, d_o, lv, pr, 0.5)
        eps = 1e-6
        for x, g in ((q, dq), (k, dk), (v, dv)):
            num = np.zeros_like(x)
            it = np.nditer(x, flags=["multi_index"])
            for _ in it:
                idx = it.multi_index
                old = x[idx]
                x[idx] = old + eps
                lp = _loss(oracle, q, k, v, d_o, lv, pr, 0.5)
                x[idx] = old - eps
                lm = _loss(oracle, q, k, v, d_o, lv, pr, 0.5)
                x[idx] = old
                num[idx] = (lp - lm) / (2 * eps)
            np.testing.assert_allclose(g, num, rtol=2e-6, atol=2e-8)
