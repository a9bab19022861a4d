"""GPU parity: decoder cross-attention over a level subset of the encoder positions (paper Sec. 4.2) against
the oracle: the two schedules bit-exact, forward and backward element by element (tolerances as for
self-attention: bf16 2e-2 on O and 5e-2 relative on gradients, fp32 1e-4)."""
import numpy as np
import pytest

from paper_2407_08330_amd import inputs
from gpu_common import GuardedWorkspace, from_dev, say, to_dev_bf16, to_dev_i32

pytestmark = pytest.mark.gpu

SEC, SENT, TOK = 1 << 1, 1 << 2, 1 << 3


def _encoder_levels(n_enc, seeds):
    """Encoder documents with the benchmark's structure, padded to n_enc."""
    lv = []
    for s in seeds:
        l, _ = inputs.tree_document([(2, 6), (2, 9), (4, 30)], np.random.default_rng(s), max_nodes=n_enc - s % 7)
        lv.append(np.concatenate([l, np.full(n_enc - l.shape[0], -1, np.int32)]))
    return np.stack(lv)


def _long_encoder_levels(n_enc, seeds, fill=1.0):
    """Documents of sections of 3..10 sentences of 5..60 tokens that fill about `fill` of n_enc positions."""
    lv = []
    for s in seeds:
        rng = np.random.default_rng(s)
        sections, used = [], 1
        while True:
            sec = [int(x) for x in rng.integers(5, 61, size=int(rng.integers(3, 11)))]
            need = 1 + sum(1 + l for l in sec)
            if used + need > int(n_enc * fill):
                break
            sections.append(sec)
            used += need
        lv.append(inputs.document_from_sections(sections, n_enc)[0])
    return np.stack(lv)


def _compare_schedule(got_layout, ref, b, what):
    got = got_layout.export(b)
    assert "kperm" not in got
    np.testing.assert_array_equal(got["q_rowptr"], ref.q_rowptr, err_msg=f"{what} q_rowptr sample {b}")
    np.testing.assert_array_equal(got["q_keys"], ref.q_keys, err_msg=f"{what} q_keys sample {b}")
    np.testing.assert_array_equal(got["q_sub"], ref.q_sub, err_msg=f"{what} q_sub sample {b}")
    np.testing.assert_array_equal(got["bits"], ref.bits, err_msg=f"{what} bits sample {b}")
    ordinal = np.arange(ref.q_keys.shape[0]) - np.repeat(ref.q_rowptr[:-1], np.diff(ref.q_rowptr))
    np.testing.assert_array_equal(got["q_cols"], ordinal)
    assert got_layout.sample_info(b) == (ref.q_keys.shape[0], ref.nnz)


@pytest.mark.parametrize("bm,bn", [(128, 64), (64, 32), (32, 32), (96, 64)])
@pytest.mark.parametrize("level_mask", [SEC, SEC | SENT, SEC | SENT | TOK, 1 | SEC, 1 << 7])
def test_cross_schedules_bit_exact(oracle, bm, bn, level_mask):
    import paper_2407_08330_amd as hdt
    n_enc, n_dec = 1000, 333
    level = _encoder_levels(n_enc, (3, 4, 5))
    level[2, :] = -1 if level_mask == SEC else level[2, :]   # one sample without any visible position
    say(f"[cross layout] {bm}x{bn} level_mask={level_mask} visible {[int(oracle.cross_select(l, level_mask).size) for l in level]}")
    lay = hdt.hdt_build_cross_layout(to_dev_i32(level), n_dec, level_mask, tile_m=bm, tile_n=bn)
    info = lay.info()
    assert (info["n_pos"], info["n_kv"], info["cross"], info["cross_level_mask"]) == (n_dec, n_enc, 1, level_mask)
    tr = lay.transposed()
    assert tr is not None
    tinfo = tr.info()
    assert (tinfo["n_pos"], tinfo["n_kv"]) == (n_enc, n_dec)
    for b in range(level.shape[0]):
        f_ref, t_ref = oracle.cross_schedule(level[b], n_dec, level_mask, bm, bn)
        _compare_schedule(lay, f_ref, b, "forward")
        _compare_schedule(tr, t_ref, b, "transposed")
        assert lay.sample_info(b)[1] == tr.sample_info(b)[1]
    # a cross layout has no key order to export
    import ctypes
    buf = np.zeros(max(n_dec, n_enc), np.int32)
    status = hdt.load_library().hdt_layout_export(lay.handle, 0, ctypes.c_void_p(buf.ctypes.data), None, None, None,
                                                  None, None, None, None, None, 0)
    assert hdt.load_library().hdt_status_string(status) == b"HDT_ERR_UNSUPPORTED"


def _tensors(B, H, n_dec, n_enc, D, seed, dtype):
    import torch
    rng = np.random.default_rng(seed)
    xs = [rng.standard_normal((B, H, n, D)).astype(np.float32) for n in (n_dec, n_enc, n_enc, n_dec)]
    if dtype == "bf16":
        xs = [inputs.round_to_bf16(x) for x in xs]
        dev = [to_dev_bf16(x) for x in xs]
    else:
        dev = [torch.from_numpy(x).cuda() for x in xs]
    return xs, dev


def pieces_of(hdt, lay, H, D, tile_m):
    """Into how many pieces the library cuts the key lists of this layout for H heads (from the size of the
    forward workspace: partial O rows of D bf16 and a partial LSE per row)."""
    need = hdt.hdt_attn_fwd_workspace_bytes(lay, H, D, 0)
    if need == 0:
        return 1
    rows_per_piece = lay.batch * H * ((lay.n_pos + tile_m - 1) // tile_m) * tile_m
    for p in (2, 4, 8):
        rows = rows_per_piece * p
        if need == ((rows * D * 2 + 255) // 256 + (rows * 4 + 255) // 256) * 256:
            return p
    raise AssertionError(f"unexpected workspace size {need}")


def run_cross_case(oracle, level, n_dec, level_mask, H, D, dtype, seed, tile=(0, 0), backward=True, want_pieces=None,
                   poison_invisible=False):
    import torch
    import paper_2407_08330_amd as hdt
    B, n_enc = level.shape
    scale = 1.0 / np.sqrt(D)
    (q, k, v, d_o), (q_, k_, v_, do_) = _tensors(B, H, n_dec, n_enc, D, seed, dtype)
    if poison_invisible:
        # K, V rows of the encoder positions the decoder does not see (pads and levels outside the mask) hold NaN and
        # infinities on the device; the oracle keeps the finite values (it never reads those rows)
        hidden = np.stack([~np.isin(np.arange(n_enc), oracle.cross_select(l, level_mask)) for l in level])
        junk = np.random.default_rng(seed).choice(np.array([np.nan, np.inf, -np.inf], np.float32), size=(B, H, n_enc, D))
        w = np.broadcast_to(hidden[:, None, :, None], k.shape)
        kd, vd = np.where(w, junk, k), np.where(w, junk[..., ::-1], v)
        k_, v_ = (to_dev_bf16(x) if dtype == "bf16" else torch.from_numpy(np.ascontiguousarray(x)).cuda() for x in (kd, vd))
    lay = hdt.hdt_build_cross_layout(to_dev_i32(level), n_dec, level_mask, tile_m=tile[0], tile_n=tile[1])
    # the backward runs on compact copies of K and V iff at most a quarter of the positions are visible
    c_max = max(int(oracle.cross_select(l, level_mask).size) for l in level)
    compact_rows = lay.info()["compact_rows"]
    say(f"    visible at most {c_max} of {n_enc}: compact rows {compact_rows}")
    assert (compact_rows > 0) == (0 < c_max and 4 * c_max <= n_enc) and (compact_rows == 0 or c_max <= compact_rows < c_max + 32)
    o_ = torch.full_like(q_, float("nan"))
    lse_ = torch.full((B, H, n_dec), float("nan"), dtype=torch.float32, device="cuda")
    # with a workspace the forward cuts long key lists into pieces (none for short lists or fp32)
    ws_bytes = hdt.hdt_attn_fwd_workspace_bytes(lay, H, D, 0 if dtype == "bf16" else 1)
    pieces = pieces_of(hdt, lay, H, D, tile[0] or 128) if dtype == "bf16" else 1
    say(f"    key lists in {pieces} piece(s), forward workspace {ws_bytes} bytes")
    assert want_pieces is None or pieces == want_pieces
    gws = GuardedWorkspace(ws_bytes) if ws_bytes else None   # exactly what the library asks for, a guard behind it
    ws = gws.view if gws else None
    hdt.hdt_attn_fwd(lay, q_, k_, v_, scale, o=o_, lse=lse_, workspace=ws)
    torch.cuda.synchronize()
    if gws:
        gws.check()
    if ws is not None:   # the same call without a workspace walks the whole lists: same result up to rounding
        o1, lse1 = hdt.hdt_attn_fwd(lay, q_, k_, v_, scale)
        torch.cuda.synchronize()
        assert np.abs(from_dev(o1) - from_dev(o_)).max() <= 2e-2
        fin = np.isfinite(lse1.cpu().numpy())
        assert np.array_equal(fin, np.isfinite(lse_.cpu().numpy()))
        assert np.abs(lse1.cpu().numpy()[fin] - lse_.cpu().numpy()[fin]).max() <= 1e-3
    o_ref, lse_ref = oracle.cross_attn_fwd(q, k, v, level, level_mask, scale)
    o_g, lse_g = from_dev(o_), lse_.cpu().numpy()
    tol_o, tol_l, tol_g = {"bf16": (2e-2, 1e-2, 5e-2), "f32": (1e-4, 1e-4, 1e-4)}[dtype]
    assert not np.isnan(o_g).any() and not np.isnan(lse_g).any()
    blind = np.array([oracle.cross_select(l, level_mask).size == 0 for l in level])
    assert (o_g[blind] == 0).all() and np.isneginf(lse_g[blind]).all()
    err_o = np.abs(o_g - o_ref).max()
    err_l = np.abs(lse_g[~blind] - lse_ref[~blind]).max() if (~blind).any() else 0.0
    say(f"    max|dO|={err_o:.3e} (tol {tol_o})  max|dLSE|={err_l:.3e} (tol {tol_l})")
    assert err_o <= tol_o and err_l <= tol_l
    if not backward:
        return
    dq_ = torch.full_like(q_, float("nan"))
    dk_ = torch.full_like(k_, float("nan"))
    dv_ = torch.full_like(k_, float("nan"))
    bws = GuardedWorkspace(hdt.hdt_attn_bwd_workspace_bytes(lay, H, D, 0 if dtype == "bf16" else 1))
    hdt.hdt_attn_bwd(lay, q_, k_, v_, o_, lse_, do_, scale, dq=dq_, dk=dk_, dv=dv_, workspace=bws.view)
    torch.cuda.synchronize()
    bws.check()
    ref = oracle.cross_attn_bwd(q, k, v, d_o, level, level_mask, scale)
    for name, g_dev, g_ref in zip(("dq", "dk", "dv"), (dq_, dk_, dv_), ref):
        g = from_dev(g_dev)
        assert not np.isnan(g).any(), f"{name}: unwritten or NaN rows"
        assert (g[g_ref == 0] == 0).all() or name == "dq", f"{name}: rows of invisible positions must be 0"
        denom = np.abs(g_ref).max()
        rel = np.abs(g - g_ref).max() / denom if denom > 0 else np.abs(g).max()
        say(f"    {name}: max-rel {rel:.3e} (tol {tol_g})")
        assert rel <= tol_g


@pytest.mark.parametrize("dtype,D", [("bf16", 64), ("bf16", 128), ("f32", 64)])
@pytest.mark.parametrize("level_mask", [SEC, SEC | SENT, SEC | SENT | TOK], ids=["sec", "sec+sent", "sec+sent+tokens"])
def test_cross_attention_ragged(oracle, dtype, D, level_mask):
    level = _encoder_levels(1000, (13, 14))
    say(f"[cross] n_enc=1000 n_dec=333 {dtype} d={D} level_mask={level_mask}")
    run_cross_case(oracle, level, 333, level_mask, 3, D, dtype, 700 + level_mask)


@pytest.mark.parametrize("tile", [(64, 32), (128, 64)], ids=["64x32", "128x64"])
def test_cross_attention_both_tile_shapes_and_blind_sample(oracle, tile):
    level = _encoder_levels(777, (23, 24, 25))
    level[1, :] = -1   # all pads: nothing visible for sample 1
    say(f"[cross] tile {tile}: n_enc=777 n_dec=130, a sample without visible positions")
    run_cross_case(oracle, level, 130, SEC | SENT, 2, 64, "bf16", 801, tile=tile)
    run_cross_case(oracle, level, 1, SEC | SENT | TOK, 2, 128, "bf16", 802, tile=tile)


@pytest.mark.parametrize("D", [64, 128])
def test_cross_attention_more_decoder_rows_than_encoder_positions(oracle, D):
    # more row tiles on the decoder side than on the encoder side: the backward's leftover workgroups are dQ roles
    level = _encoder_levels(150, (33, 34))
    say(f"[cross] n_enc=150 n_dec=1000 d={D}")
    run_cross_case(oracle, level, 1000, SEC | SENT | TOK, 2, D, "bf16", 850 + D)
    run_cross_case(oracle, level, 1000, SEC, 2, D, "bf16", 860 + D, tile=(64, 32))


def test_cross_attention_benchmark_documents(oracle):
    # the encoder side of the benchmark's 8192-position batch; 512 decoder rows (section-level summaries)
    wl = inputs.make_workload(4)
    for level_mask in (SEC, SEC | SENT, SEC | SENT | TOK):
        say(f"[cross] config 4 documents, n_dec=512, level_mask={level_mask}: visible "
            f"{[int(oracle.cross_select(l, level_mask).size) for l in wl.level]}")
        run_cross_case(oracle, wl.level, 512, level_mask, 4, 64, "bf16", 900 + level_mask)


@pytest.mark.parametrize("D", [64, 128])
def test_cross_attention_long_key_lists_cut_into_pieces(oracle, D):
    # the regular tokens visible and few decoder rows: a handful of row tiles with lists of dozens of entries, which
    # the library cuts into pieces walked by separate workgroups (forward with a workspace; dQ role of the backward)
    level = _long_encoder_levels(5000, (43,))
    say(f"[cross] n_enc=5000 n_dec=100, tokens visible, d={D}: 8 pieces")
    run_cross_case(oracle, level, 100, SEC | SENT | TOK, 2, D, "bf16", 950 + D, want_pieces=8)
    level = _long_encoder_levels(3000, (44, 45))
    level[1, 1500:] = -1   # the second sample sees half as much: its later pieces are empty
    say(f"[cross] n_enc=3000 n_dec=333 (a ragged last row tile), tokens visible, d={D}: 4 pieces")
    run_cross_case(oracle, level, 333, SEC | SENT | TOK, 3, D, "bf16", 960 + D, want_pieces=4)
    say(f"[cross] the same at 64x32 tiles")
    run_cross_case(oracle, level, 333, SEC | SENT | TOK, 3, D, "bf16", 970 + D, tile=(64, 32))
    # short lists, and fp32: nothing to cut
    run_cross_case(oracle, _encoder_levels(600, (46,)), 100, SEC | SENT | TOK, 2, D, "bf16", 980 + D, want_pieces=1)
    run_cross_case(oracle, _long_encoder_levels(3000, (47,)), 64, SEC | SENT | TOK, 1, D, "f32", 990 + D, want_pieces=1, backward=False)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_cross_attention_ignores_what_invisible_rows_hold(oracle, dtype):
    # pads in front and behind, NaN / Inf in every K, V row the level mask hides: anchors only (the backward works on
    # compact copies), and everything but [DOC] (the backward tiles the encoder rows, hidden ones among them)
    level = _long_encoder_levels(1536, (51, 52), fill=0.8)
    level = np.concatenate([np.full((2, 40), -1, np.int32), level[:, :-40]], axis=1)
    for level_mask in (SEC | SENT, SEC | SENT | TOK):
        say(f"[cross] NaN/Inf in hidden K, V rows, level_mask={level_mask}, {dtype}")
        run_cross_case(oracle, level, 200, level_mask, 2, 64, dtype, 1000 + level_mask, poison_invisible=True)


def test_cross_argument_errors():
    import torch
    import paper_2407_08330_amd as hdt
    level = to_dev_i32(_encoder_levels(256, (1,)))
    with pytest.raises(hdt.HdtError) as e:
        hdt.hdt_build_cross_layout(level, 64, SEC, tile_m=48)
    assert e.value.name == "HDT_ERR_UNSUPPORTED"
    with pytest.raises(hdt.HdtError) as e:
        hdt.hdt_build_cross_layout(level, -1, SEC)
    assert e.value.name == "HDT_ERR_INVALID_ARG"
    lay = hdt.hdt_build_cross_layout(level, 64, SEC)
    q = torch.zeros((1, 2, 64, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ValueError):
        hdt.hdt_attn_fwd(lay, q, q.clone(), q.clone(), 0.1)   # k, v must have the encoder's length
    for n_enc, n_dec in ((0, 64), (256, 0)):   # both sides need rows
        lv = torch.zeros((1, n_enc), dtype=torch.int32, device="cuda")
        with pytest.raises(hdt.HdtError) as e:
            hdt.hdt_build_cross_layout(lv, n_dec, 1)
        assert e.value.name == "HDT_ERR_SHAPE"
    lay0 = hdt.hdt_build_cross_layout(torch.zeros((0, 256), dtype=torch.int32, device="cuda"), 64, 1)
    assert lay0.info()["n_tiles"] == 0 and lay0.transposed().info()["n_tiles"] == 0
