"""GPU parity with non-finite values where the mask says nothing may be read (Sec. 3.2: a masked pair
contributes nothing).  Pad rows of Q, K, V, dO are filled with NaN and +-Inf: every result must be what it is
with finite pads (the oracle never reads a pad row), pad rows of O and of the gradients must be 0 and of LSE
-inf.  A second case poisons the K, V rows of a few REAL positions and looks at the rows of query tiles in
which no row may attend to them: those results must not move either (a windowed layout gathers whole windows
of the key order, so such rows do sit in the gathered tiles).  Tolerances are the contract's."""
import numpy as np
import pytest

from paper_2407_08330_amd import inputs
from gpu_common import from_dev, say, to_dev_bf16, to_dev_i32

pytestmark = pytest.mark.gpu

TOL_FWD = {"bf16": (2e-2, 1e-2), "f32": (1e-4, 1e-4)}
TOL_BWD = {"bf16": 5e-2, "f32": 1e-4}


def padded_documents(n_pos, front, seed, n_sec=3, n_sent=4):
    """Two samples: a config-1-like document with `front` pads in front of it and pads behind, and a
    ListOps-shaped tree with pads behind only."""
    rng = np.random.default_rng(seed)
    lens = [[int(x) for x in rng.integers(5, 40, size=n_sent)] for _ in range(n_sec)]
    n_doc = 1 + sum(1 + sum(1 + l for l in sec) for sec in lens)
    lv, pr = inputs.document_from_sections(lens, n_doc)
    lv0 = np.full(n_pos, -1, np.int32)
    pr0 = np.full(n_pos, -1, np.int32)
    lv0[front:front + n_doc] = lv
    pr0[front:front + n_doc] = np.where(pr >= 0, pr + front, -1)
    lv1, pr1 = inputs.listops_like_tree(rng, n_pos, max_depth=8, max_nodes=n_pos - 97)
    return np.stack([lv0, lv1]), np.stack([pr0, pr1])


def poison(x, where, kind, rng):
    """x [B][H][N][D] float32; rows where[b][n] get NaN / +-Inf / a mix."""
    y = x.copy()
    B, H, N, D = x.shape
    w = np.broadcast_to(where[:, None, :, None], x.shape)
    if kind == "nan":
        y[w] = np.nan
    elif kind == "inf":
        y[w] = np.where(rng.random(int(w.sum())) < 0.5, np.inf, -np.inf)
    else:
        y[w] = rng.choice(np.array([np.nan, np.inf, -np.inf, 3.0e38], np.float32), size=int(w.sum()))
    return y


def to_dev(x, dtype):
    import torch
    if dtype == "bf16":
        return to_dev_bf16(x)   # NaN and Inf have exact bf16 forms (the upper 16 bits)
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def run_all(hdt, lay, tensors, dtype, scale):
    import torch
    q_, k_, v_, do_ = (to_dev(x, dtype) for x in tensors)
    o_ = torch.full_like(q_, float("nan"))
    lse_ = torch.full(q_.shape[:3], float("nan"), dtype=torch.float32, device="cuda")
    hdt.hdt_attn_fwd(lay, q_, k_, v_, scale, o=o_, lse=lse_)
    dq_, dk_, dv_ = (torch.full_like(q_, float("nan")) for _ in range(3))
    hdt.hdt_attn_bwd(lay, q_, k_, v_, o_, lse_, do_, scale, dq=dq_, dk=dk_, dv=dv_)
    torch.cuda.synchronize()
    return from_dev(o_), lse_.cpu().numpy(), from_dev(dq_), from_dev(dk_), from_dev(dv_)


@pytest.mark.parametrize("kind", ["nan", "inf", "mixed"])
@pytest.mark.parametrize("windowed", [False, True])
@pytest.mark.parametrize("tile", [(128, 64), (64, 32)])
@pytest.mark.parametrize("dtype,D", [("bf16", 64), ("bf16", 128), ("f32", 64)])
def test_nonfinite_pad_rows_change_nothing(oracle, kind, windowed, tile, dtype, D):
    import paper_2407_08330_amd as hdt
    N, H = 640, 2
    level, parent = padded_documents(N, front=37, seed=4242)
    B = level.shape[0]
    scale = 1.0 / np.sqrt(D)
    clean = inputs.make_qkv(B, H, N, D, 9001, 4)
    if dtype == "bf16":
        clean = [inputs.round_to_bf16(x) for x in clean]
    rng = np.random.default_rng(7)
    pad = level < 0
    dirty = [poison(x, pad, kind, rng) for x in clean]
    say(f"[nonfinite] pads = {kind}, {'windowed' if windowed else 'key lists'}, tile {tile}, {dtype} d={D}")
    lay = hdt.hdt_build_layout(to_dev_i32(level), to_dev_i32(parent), tile_m=tile[0], tile_n=tile[1], windowed=windowed)
    o, lse, dq, dk, dv = run_all(hdt, lay, dirty, dtype, scale)
    o_ref, lse_ref = oracle.attn_fwd(*clean[:3], level, parent, scale)
    g_ref = oracle.attn_bwd(*clean, level, parent, scale)
    padr = np.broadcast_to(pad[:, None, :, None], o.shape)
    padl = np.broadcast_to(pad[:, None, :], lse.shape)
    for name, g in (("o", o), ("dq", dq), ("dk", dk), ("dv", dv)):
        assert np.isfinite(g).all(), f"{name}: non-finite values leaked out of pad rows"
        assert (g[padr] == 0).all(), f"{name}: pad rows must be 0"
    assert np.isneginf(lse[padl]).all() and np.isfinite(lse[~padl]).all()
    tol_o, tol_l = TOL_FWD[dtype]
    err_o, err_l = np.abs(o - o_ref).max(), np.abs(lse[~padl] - lse_ref[~padl]).max()
    say(f"    max|dO|={err_o:.3e} max|dLSE|={err_l:.3e}")
    assert err_o <= tol_o and err_l <= tol_l
    for name, g, r in zip(("dq", "dk", "dv"), (dq, dk, dv), g_ref):
        rel = np.abs(g - r).max() / np.abs(r).max()
        say(f"    {name}: max-rel {rel:.3e}")
        assert rel <= TOL_BWD[dtype]
    lay.destroy()


@pytest.mark.parametrize("windowed", [False, True])
@pytest.mark.parametrize("tile", [(128, 64), (64, 32)])
def test_nonfinite_real_rows_stay_inside_the_tiles_that_attend_to_them(oracle, windowed, tile):
    """K, V rows of a few real positions are NaN.  A row of a query tile in which NO row may attend to a
    poisoned position must come out as with clean inputs: such keys are in no key list, and where a window of
    the key order holds them the library gathers another row in their place.  (Rows of tiles that do gather a
    poisoned key may turn NaN: its zero weights are applied by multiplication.)"""
    import paper_2407_08330_amd as hdt
    N, H, D, dtype = 2048, 2, 64, "bf16"
    bm = tile[0]
    level, parent = padded_documents(N, front=5, seed=99, n_sec=6, n_sent=6)
    B = level.shape[0]
    scale = 1.0 / np.sqrt(D)
    clean = [inputs.round_to_bf16(x) for x in inputs.make_qkv(B, H, N, D, 9100, 4)]
    rng = np.random.default_rng(11)
    M = np.stack([oracle.mask(level[b], parent[b]).astype(bool) for b in range(B)])   # [B][N][N]
    bad = np.zeros((B, N), bool)
    for b in range(B):
        real = np.flatnonzero(level[b] >= 0)
        # leaves of the hierarchy only (nobody's parent): an anchor is seen from too many tiles to leave a test
        leaves = np.setdiff1d(real, parent[b][real])
        bad[b, rng.choice(leaves, size=2, replace=False)] = True
    dirty = [clean[0], poison(clean[1], bad, "nan", rng), poison(clean[2], bad, "nan", rng), clean[3]]
    # rows whose query tile holds a row that may attend to a poisoned key (forward, dQ: O, LSE, D of all rows of
    # such a tile may be NaN), and the keys whose tile of key rows holds a key that such a row may attend to (dK,
    # dV: the backward tiles the keys the same way and gathers the query rows)
    tile_hit = np.zeros((B, N), bool)
    for b in range(B):
        hit_rows = M[b][:, bad[b]].any(axis=1)
        for I in range(N // bm):
            if hit_rows[I * bm:(I + 1) * bm].any():
                tile_hit[b, I * bm:(I + 1) * bm] = True
    key_hit = np.stack([M[b][tile_hit[b]].any(axis=0) for b in range(B)])
    for b in range(B):
        for I in range(N // bm):
            if key_hit[b, I * bm:(I + 1) * bm].any():
                key_hit[b, I * bm:(I + 1) * bm] = True
    say(f"[nonfinite] 2 NaN keys per sample, {'windowed' if windowed else 'key lists'}, tile {tile}: "
        f"{int(tile_hit.sum())} rows and {int(key_hit.sum())} keys may be touched, of {int((level >= 0).sum())}")
    # enough of the documents is left to look at
    assert (~tile_hit & (level >= 0)).sum() >= 500 and (~key_hit & (level >= 0)).sum() >= 100
    lay = hdt.hdt_build_layout(to_dev_i32(level), to_dev_i32(parent), tile_m=tile[0], tile_n=tile[1], windowed=windowed)
    o, lse, dq, dk, dv = run_all(hdt, lay, dirty, dtype, scale)
    o_ref, lse_ref = oracle.attn_fwd(*clean[:3], level, parent, scale)
    dq_ref, dk_ref, dv_ref = oracle.attn_bwd(*clean, level, parent, scale)
    rows = np.broadcast_to((~tile_hit)[:, None, :, None], o.shape)
    keys = np.broadcast_to((~key_hit)[:, None, :, None], o.shape)
    rows_l = np.broadcast_to((~tile_hit & (level >= 0))[:, None, :], lse.shape)
    assert np.abs(o[rows] - o_ref[rows]).max() <= 2e-2
    assert np.abs(lse[rows_l] - lse_ref[rows_l]).max() <= 1e-2
    assert np.abs(dq[rows] - dq_ref[rows]).max() / np.abs(dq_ref).max() <= 5e-2
    assert np.abs(dk[keys] - dk_ref[keys]).max() / np.abs(dk_ref).max() <= 5e-2
    assert np.abs(dv[keys] - dv_ref[keys]).max() / np.abs(dv_ref).max() <= 5e-2
    lay.destroy()
