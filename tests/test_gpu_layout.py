"""GPU parity: hdt_build_layout against the oracle's brute-force schedules, bit-exact: the
per-query-tile key lists (the default) and the windowed block schedule of Alg. 1."""
import numpy as np
import pytest

from paper_2407_08330_amd import inputs
from gpu_common import compare_layout, say, to_dev_i32

pytestmark = pytest.mark.gpu


def _build(level, parent, **kw):
    import paper_2407_08330_amd as hdt
    return hdt.hdt_build_layout(to_dev_i32(level), to_dev_i32(parent), **kw)


WINDOWED = pytest.mark.parametrize("windowed", [False, True], ids=["keylists", "windowed"])


@WINDOWED
@pytest.mark.parametrize("config", [1, 2, 3, 5])
def test_layout_matches_oracle_on_benchmark_configs(oracle, config, windowed):
    wl = inputs.make_workload(config)
    say(f"[layout] config {config} B={wl.batch} N={wl.n_pos} windowed={windowed}")
    lay = _build(wl.level, wl.parent, windowed=windowed)
    tiles, nnz = compare_layout(oracle, lay, wl.level, wl.parent, 128, 64, windowed=windowed)
    say(f"[layout] config {config}: {tiles} tiles, nnz {nnz}")
    lay.destroy()


@pytest.mark.parametrize("config", [3, 5])
def test_layout_64x32_on_benchmark_configs(oracle, config):
    wl = inputs.make_workload(config)
    say(f"[layout] config {config} B={wl.batch} N={wl.n_pos} tile 64x32")
    lay = _build(wl.level, wl.parent, tile_m=64, tile_n=32)
    tiles, nnz = compare_layout(oracle, lay, wl.level, wl.parent, 64, 32)
    say(f"[layout] config {config}: {tiles} tiles, nnz {nnz}")
    lay.destroy()


@WINDOWED
@pytest.mark.parametrize("bm,bn", [(64, 32), (32, 32), (128, 128), (96, 64), (64, 64), (64, 128), (32, 96)])
def test_layout_other_tile_shapes(oracle, bm, bn, windowed):
    wl = inputs.make_workload(2, batch=2)
    say(f"[layout] tile {bm}x{bn} windowed={windowed}")
    lay = _build(wl.level, wl.parent, tile_m=bm, tile_n=bn, windowed=windowed)
    compare_layout(oracle, lay, wl.level, wl.parent, bm, bn, windowed=windowed)


@WINDOWED
@pytest.mark.parametrize("bm,bn", [(128, 64), (64, 32)])
@pytest.mark.parametrize("n", [1, 31, 100, 129, 1000, 4097])
def test_layout_ragged_lengths(oracle, n, bm, bn, windowed):
    # 64-row tiles: an odd number of query tiles at 31, 129 and 4097 (key lists of two neighbouring tiles are
    # built by one workgroup, the last one then has a single tile)
    rng = np.random.default_rng(n)
    level, parent = inputs.tree_document([(1, 6), (0, 7), (0, 20)], rng, max_nodes=n)
    level = np.concatenate([level, np.full(n - level.shape[0], -1, np.int32)])[None]
    parent = np.concatenate([parent, np.full(n - parent.shape[0], -1, np.int32)])[None]
    say(f"[layout] ragged n={n} real={(level >= 0).sum()} tile {bm}x{bn} windowed={windowed}")
    lay = _build(level, parent, tile_m=bm, tile_n=bn, windowed=windowed)
    compare_layout(oracle, lay, level, parent, bm, bn, windowed=windowed)


@WINDOWED
def test_layout_deep_trees_and_all_pad_sample(oracle, windowed):
    rng = np.random.default_rng(11)
    n = 768
    lv, pr = [], []
    for s in range(3):
        l, p = inputs.tree_document([(1, 4)] * 7 + [(0, 5)], rng, n_pos=None, max_nodes=n)
        lv.append(np.concatenate([l, np.full(n - l.shape[0], -1, np.int32)]))
        pr.append(np.concatenate([p, np.full(n - p.shape[0], -1, np.int32)]))
    lv.append(np.full(n, -1, np.int32))   # an empty document: all pads
    pr.append(np.full(n, -1, np.int32))
    level, parent = np.stack(lv), np.stack(pr)
    say(f"[layout] deep trees + all-pad sample windowed={windowed}")
    lay = _build(level, parent, windowed=windowed)
    compare_layout(oracle, lay, level, parent, 128, 64, windowed=windowed)
    assert lay.sample_info(3) == (0, 0)


@WINDOWED
def test_layout_positions_not_in_preorder(oracle, windowed):
    # a shuffled document: sibling groups are scattered, the marked ranges over-approximate and the
    # exact evaluation has to drop the empty windows / the keys no row of the tile attends to
    wl = inputs.make_workload(1)
    rng = np.random.default_rng(5)
    n = wl.n_pos
    perm = rng.permutation(n)              # new position of old position i is perm[i]
    level = np.empty(n, np.int32)
    parent = np.empty(n, np.int32)
    level[perm] = wl.level[0]
    old_parent = wl.parent[0]
    parent[perm] = np.where(old_parent >= 0, perm[np.maximum(old_parent, 0)], -1)
    say(f"[layout] shuffled positions windowed={windowed}")
    lay = _build(level[None], parent[None], windowed=windowed)
    compare_layout(oracle, lay, level[None], parent[None], 128, 64, windowed=windowed)


def test_layout_force_dense_and_no_sort(oracle):
    wl = inputs.make_workload(1)
    say("[layout] force_dense / no_sort")
    lay = _build(wl.level, wl.parent, force_dense=True)
    tiles, _ = compare_layout(oracle, lay, wl.level, wl.parent, 128, 64, force_dense=True)
    assert tiles == 4 * 8
    for windowed in (True, False):
        lay = _build(wl.level, wl.parent, no_sort=True, windowed=windowed)
        compare_layout(oracle, lay, wl.level, wl.parent, 128, 64, windowed=windowed, use_sort=False)


@pytest.mark.parametrize("bm,bn", [(128, 64), (64, 32), (96, 128), (64, 128), (32, 64)])
@pytest.mark.parametrize("n_children", [1500, 2999])
def test_layout_one_parent_with_thousands_of_children(oracle, n_children, bm, bn):
    # every tile's key list holds the root and all its children: 1501 keys still fit the kernel's on-chip copy
    # of a list (several rounds of entries), 3000 do not (the list goes through global memory); sample 1 is an
    # ordinary document, so both kinds of tile meet in one launch
    n = 3072
    level = np.full((2, n), -1, np.int32)
    parent = np.full((2, n), -1, np.int32)
    level[0, 0] = 0
    level[0, 1:1 + n_children] = 1
    parent[0, 1:1 + n_children] = 0
    wl = inputs.make_workload(1, batch=1)
    level[1, :wl.n_pos] = wl.level[0]
    parent[1, :wl.n_pos] = wl.parent[0]
    say(f"[layout] root with {n_children} children, tile {bm}x{bn}")
    lay = _build(level, parent, tile_m=bm, tile_n=bn)
    tiles, nnz = compare_layout(oracle, lay, level, parent, bm, bn)
    assert nnz >= (n_children + 1) ** 2


@pytest.mark.parametrize("log2n,n_sections,bm,bn", [(17, 120, 128, 64), (19, 500, 128, 64), (17, 120, 64, 32)])
def test_layout_long_documents_need_a_large_slot_bitmap(oracle, log2n, n_sections, bm, bn):
    # 2^17 / 2^19 (the largest accepted) positions: the key-list kernel's bitmaps over the positions take
    # 32 KB / 128 KB of LDS; with 64-row tiles two such sets no longer fit one workgroup, and every tile gets a
    # workgroup of its own (512 threads)
    rng = np.random.default_rng(77)
    n = 1 << log2n
    secs = [[int(rng.integers(5, 61)) for _ in range(int(rng.integers(5, 41)))] for _ in range(n_sections)]
    level, parent = inputs.document_from_sections(secs, n)
    say(f"[layout] n = {n}, real = {(level >= 0).sum()}, tile {bm}x{bn}")
    lay = _build(level[None], parent[None], tile_m=bm, tile_n=bn)
    got = lay.export(0)
    ref_kperm = oracle.kperm(level)
    np.testing.assert_array_equal(got["kperm"], ref_kperm)
    # the full brute force is n^2; check sampled query tiles against the oracle's pair test instead
    rowptr = got["q_rowptr"]
    slot = np.empty(n, np.int64)
    slot[ref_kperm] = np.arange(n)
    for I in rng.choice(n // bm, size=12, replace=False).tolist() + [0]:
        rows = np.arange(I * bm, (I + 1) * bm)
        keys = got["q_keys"][rowptr[I]:rowptr[I + 1]].reshape(-1)
        real = keys[keys >= 0]
        assert (keys[len(real):] == -1).all() and (np.diff(slot[real]) > 0).all()
        want = set()
        for i in rows:
            if level[i] < 0:
                continue
            cand = {int(i)} | ({int(parent[i])} if parent[i] >= 0 else set())
            cand |= set(np.nonzero(parent == i)[0].tolist())
            if parent[i] >= 0:
                cand |= set(np.nonzero(parent == parent[i])[0].tolist())
            for j in cand:
                assert oracle.allowed(level, parent, int(i), j)
            want |= cand
        assert set(real.tolist()) == want, f"query tile {I}"
        bits = got["bits"][rowptr[I]:rowptr[I + 1]]
        for e in range(bits.shape[0]):
            for c in range(bn):
                j = keys[e * bn + c]
                col = (bits[e, :, c // 32] >> np.uint32(c % 32)) & 1
                exp = [oracle.allowed(level, parent, int(i), int(j)) if j >= 0 else 0 for i in rows]
                np.testing.assert_array_equal(col, np.array(exp, np.uint32))


@WINDOWED
@pytest.mark.parametrize("edges", [2 | 4, 4, 1 | 2, 1, 2], ids=["green+blue", "blue", "up+sibling", "up", "sibling"])
def test_layout_listops_mask_variants(oracle, edges, windowed):
    # thinned / directed masks (paper Sec. 4.1) on ListOps-shaped trees and on a document
    rng = np.random.default_rng(99)
    lv, pr = inputs.listops_like_tree(rng, 1000)
    wl = inputs.make_workload(1)
    for level, parent in ((lv[None], pr[None]), (wl.level, wl.parent)):
        say(f"[layout] edges={edges} windowed={windowed} n={level.shape[1]}")
        lay = _build(level, parent, edges=edges, windowed=windowed)
        assert lay.info()["edges"] == edges
        compare_layout(oracle, lay, level, parent, 128, 64, windowed=windowed, edges=edges)
        # a directed mask also holds the schedule of its transpose (for dK, dV): the same construction with
        # the parent and child kinds exchanged; a symmetric one has none
        swapped = (edges & 2) | (4 if edges & 1 else 0) | (1 if edges & 4 else 0)
        tr = lay.transposed()
        if swapped == edges:
            assert tr is None
        else:
            assert tr.info()["edges"] == swapped
            compare_layout(oracle, tr, level, parent, 128, 64, windowed=windowed, edges=swapped)


@WINDOWED
def test_layout_grows_its_arrays_when_the_first_guess_is_too_small(oracle, windowed):
    # a dense document (one root, everything else its children) needs n/64 entries per query tile, far more
    # than the size guessed from the previous (tiny) build: the build is repeated with the exact size
    tiny_l = np.array([[0, 1, 1, -1]], np.int32)
    tiny_p = np.array([[-1, 0, 0, -1]], np.int32)
    _build(tiny_l, tiny_p, windowed=windowed).destroy()
    n = 3000
    level = np.array([[0] + [1] * (n - 1)], np.int32)
    parent = np.array([[-1] + [0] * (n - 1)], np.int32)
    say(f"[layout] dense document n={n} after a tiny one, windowed={windowed}")
    lay = _build(level, parent, windowed=windowed)
    tiles, nnz = compare_layout(oracle, lay, level, parent, 128, 64, windowed=windowed)
    assert nnz == n * n and tiles == 24 * 47
    lay.destroy()
    _build(tiny_l, tiny_p, tile_m=64, tile_n=32, windowed=windowed).destroy()
    lay = _build(level, parent, tile_m=64, tile_n=32, windowed=windowed)   # 47 query tiles: the last on its own
    tiles, nnz = compare_layout(oracle, lay, level, parent, 64, 32, windowed=windowed)
    assert nnz == n * n and tiles == 47 * 94


def test_layout_rejects_bad_hierarchies():
    import paper_2407_08330_amd as hdt
    good_l = np.array([[0, 1, 2, 3, -1, -1]], np.int32)
    good_p = np.array([[-1, 0, 1, 2, -1, -1]], np.int32)
    _build(good_l, good_p)
    cases = {
        "self parent": (good_l, np.array([[-1, 1, 1, 2, -1, -1]], np.int32)),
        "parent out of range": (good_l, np.array([[-1, 0, 1, 6, -1, -1]], np.int32)),
        "parent below -1": (good_l, np.array([[-2, 0, 1, 2, -1, -1]], np.int32)),
        "pad with parent": (good_l, np.array([[-1, 0, 1, 2, 0, -1]], np.int32)),
        "pad parent": (good_l, np.array([[-1, 0, 1, 4, -1, -1]], np.int32)),
        "level too large": (np.array([[0, 1, 2, 32, -1, -1]], np.int32), good_p),
        "level below -1": (np.array([[0, 1, 2, 3, -2, -1]], np.int32), good_p),
    }
    for name, (l, p) in cases.items():
        say(f"[layout] reject: {name}")
        with pytest.raises(hdt.HdtError) as e:
            _build(l, p)
        assert e.value.name == "HDT_ERR_HIERARCHY", name


def test_layout_many_builds_in_a_row_share_the_counter_slots(oracle):
    # a key-list build counts in one of 64 device slots that its kernel clears before it reports: 150 builds,
    # different inputs in turn and a rejected hierarchy now and then, must each see a clear slot
    import paper_2407_08330_amd as hdt
    a = inputs.make_workload(1, batch=2)
    b = inputs.make_workload(2, batch=1)
    bad_l = np.array([[0, 1, 2, 3, -1, -1]], np.int32)
    bad_p = np.array([[-1, 1, 1, 2, -1, -1]], np.int32)
    say("[layout] 150 builds in a row")
    want = {}
    for k in range(150):
        wl = a if k % 2 == 0 else b
        lay = _build(wl.level, wl.parent)
        info = lay.info()
        key = k % 2
        if key not in want:
            compare_layout(oracle, lay, wl.level, wl.parent, 128, 64)
            want[key] = (info["n_tiles"], info["nnz"])
        assert (info["n_tiles"], info["nnz"]) == want[key], f"build {k}"
        lay.destroy(completed=k % 3 == 0)   # info() has waited for the device: nothing is left to order
        if k % 37 == 5:
            with pytest.raises(hdt.HdtError):
                _build(bad_l, bad_p)
    lay = _build(b.level, b.parent)
    compare_layout(oracle, lay, b.level, b.parent, 128, 64)


def test_layout_builds_from_two_host_threads(oracle):
    # two host threads build on streams of their own at the same time (the binding releases the GIL inside the
    # call): tickets, report words, counter slots and the buffer cache are shared state of the library
    import threading
    import torch
    import paper_2407_08330_amd as hdt
    work = [inputs.make_workload(1, batch=2), inputs.make_workload(2, batch=1)]
    want = []
    for wl in work:
        lay = _build(wl.level, wl.parent)
        compare_layout(oracle, lay, wl.level, wl.parent, 128, 64)
        info = lay.info()
        want.append((info["n_tiles"], info["nnz"]))
    dev = [(to_dev_i32(wl.level), to_dev_i32(wl.parent)) for wl in work]
    errors = []

    def builder(k):
        try:
            stream = torch.cuda.Stream()
            for it in range(40):
                which = (k + it) % 2
                lay = hdt.hdt_build_layout(dev[which][0], dev[which][1], stream=stream)
                info = lay.info()
                if (info["n_tiles"], info["nnz"]) != want[which]:
                    errors.append(f"thread {k} build {it}: {info['n_tiles']}, {info['nnz']} instead of {want[which]}")
                lay.destroy()
        except Exception as e:   # noqa: BLE001 - reported below
            errors.append(f"thread {k}: {e!r}")

    say("[layout] 2 threads x 40 builds")
    threads = [threading.Thread(target=builder, args=(k,)) for k in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
        assert not t.is_alive(), "a builder thread is stuck"
    torch.cuda.synchronize()
    assert not errors, errors[:3]


def test_deferred_build_matches_the_waiting_one(oracle):
    # a deferred build only enqueues its kernel; the schedule it leaves is the same, and hdt_layout_status tells
    # how many list entries it needed
    import torch
    import paper_2407_08330_amd as hdt
    for config, tile in [(1, (128, 64)), (2, (128, 64)), (3, (64, 32))]:
        wl = inputs.make_workload(config, batch=2 if config > 1 else None)
        say(f"[layout] deferred build, config {config}, tile {tile}")
        lay = _build(wl.level, wl.parent, tile_m=tile[0], tile_n=tile[1], deferred=True)
        need = lay.status()
        tiles, _ = compare_layout(oracle, lay, wl.level, wl.parent, tile[0], tile[1])
        assert need == tiles
        lay.destroy()
    # a directed mask brings a second schedule: both builds are deferred, the status covers both
    rng = np.random.default_rng(5)
    lv, pr = inputs.listops_like_tree(rng, 1024, max_depth=12)
    edges = hdt.HDT_EDGE_SIBLING | hdt.HDT_EDGE_DOWN
    lay = _build(lv[None], pr[None], edges=edges, deferred=True)
    need = lay.status()
    t_fwd, _ = compare_layout(oracle, lay, lv[None], pr[None], 128, 64, edges=edges)
    t_tr, _ = compare_layout(oracle, lay.transposed(), lv[None], pr[None], 128, 64, edges=hdt.HDT_EDGE_SIBLING | hdt.HDT_EDGE_UP)
    assert need == max(t_fwd, t_tr)
    lay.destroy()
    # many deferred builds in a row on one stream, looked at only at the end (the report slots are a ring)
    wl = inputs.make_workload(1)
    lv, pr = to_dev_i32(wl.level), to_dev_i32(wl.parent)
    lays = [hdt.hdt_build_layout(lv, pr, deferred=True) for _ in range(40)]
    torch.cuda.synchronize()
    want = lays[0].info()
    for lay in lays:
        info = lay.info()
        assert (info["n_tiles"], info["nnz"]) == (want["n_tiles"], want["nnz"])
        lay.destroy()


def test_deferred_build_reports_its_errors_later(oracle):
    import torch
    import paper_2407_08330_amd as hdt
    bad_l = np.array([[0, 1, 2, 3, -1, -1] + [-1] * 122], np.int32)
    bad_p = np.array([[-1, 1, 1, 2, -1, -1] + [-1] * 122], np.int32)   # position 1 is its own parent
    say("[layout] deferred build of an invalid hierarchy")
    lay = _build(bad_l, bad_p, deferred=True)          # returns without having looked
    with pytest.raises(hdt.HdtError) as e:
        lay.status()
    assert e.value.name == "HDT_ERR_HIERARCHY"
    q = torch.zeros((1, 1, 128, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(hdt.HdtError) as e:               # known by now: attention calls refuse the layout
        hdt.hdt_attn_fwd(lay, q, q.clone(), q.clone(), 0.125)
    assert e.value.name == "HDT_ERR_HIERARCHY"
    with pytest.raises(hdt.HdtError):
        lay.info()
    lay.destroy()

    # too little room: the kernels stay inside the arrays, the status says how much is needed
    n = 3000
    level = np.array([[0] + [1] * (n - 1) + [-1] * 72], np.int32)
    parent = np.array([[-1] + [0] * (n - 1) + [-1] * 72], np.int32)
    say("[layout] deferred build with too small a capacity")
    x = torch.randn((1, 2, n + 72, 64), device="cuda").to(torch.bfloat16)
    y, z = x.clone(), x.clone()
    lv, pr = to_dev_i32(level), to_dev_i32(parent)
    torch.cuda.synchronize()
    lay = hdt.hdt_build_layout(lv, pr, deferred=True, capacity=100)
    try:   # enqueued right behind the build: runs on the truncated lists, inside the arrays ...
        hdt.hdt_attn_fwd(lay, x, y, z, 0.125)
    except hdt.HdtError as err:   # ... unless the report was quicker than this host thread
        assert err.name == "HDT_ERR_SHAPE"
    torch.cuda.synchronize()
    with pytest.raises(hdt.HdtError) as e:
        lay.status()
    assert e.value.name == "HDT_ERR_SHAPE" and e.value.entries_needed == 24 * 47
    lay.destroy()
    lay = _build(level, parent, deferred=True, capacity=24 * 47)
    assert lay.status() == 24 * 47 and lay.info()["nnz"] == n * n
    lay.destroy()
    # the same limit on a build that waits: an error instead of a second attempt
    with pytest.raises(hdt.HdtError) as e:
        _build(level, parent, capacity=100)
    assert e.value.name == "HDT_ERR_SHAPE"
    lay = _build(level, parent, capacity=24 * 47 + 5)
    assert lay.info()["n_tiles"] == 24 * 47
    lay.destroy()
    # 64 x 32 tiles (two query tiles per workgroup share one reservation): 47 tiles with rows x 94 entries
    for capacity in (100, 94 + 50, 47 * 94 - 1):
        lay = hdt.hdt_build_layout(lv, pr, tile_m=64, tile_n=32, deferred=True, capacity=capacity)
        try:
            hdt.hdt_attn_fwd(lay, x, y, z, 0.125)
        except hdt.HdtError as err:
            assert err.name == "HDT_ERR_SHAPE"
        torch.cuda.synchronize()
        with pytest.raises(hdt.HdtError) as e:
            lay.status()
        assert e.value.name == "HDT_ERR_SHAPE" and e.value.entries_needed == 47 * 94
        lay.destroy()
    lay = _build(level, parent, tile_m=64, tile_n=32, deferred=True, capacity=47 * 94)
    assert lay.status() == 47 * 94 and lay.info()["nnz"] == n * n
    compare_layout(oracle, lay, level, parent, 64, 32)
    lay.destroy()


def test_layout_empty_inputs():
    import torch
    import paper_2407_08330_amd as hdt
    for shape in [(0, 128), (3, 0), (0, 0)]:
        z = torch.zeros(shape, dtype=torch.int32, device="cuda")
        lay = hdt.hdt_build_layout(z, z.clone())
        info = lay.info()
        assert info["n_tiles"] == 0 and info["nnz"] == 0 and info["batch"] == shape[0]
