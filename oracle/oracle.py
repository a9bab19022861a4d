"""Python face of the CPU oracle (test infrastructure only).

Thin ctypes glue over ``hdt_oracle.c`` plus the few steps that are clearer in numpy
(assembling block lists from per-block counts).  Nothing here is imported by the product
path, and nothing here imports the product package.

Paper passages followed are cited in ``hdt_oracle.c``; the block schedule follows
App. A.1, Alg. 1 (sort keys by level, partition into M x N blocks, skip blocks whose mask
is all zero).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hdt_oracle.c")
# HDT_ORACLE_SANITIZE=1 (CPU test runs only): the oracle built with AddressSanitizer and
# UndefinedBehaviorSanitizer, loaded by a python started with gcc's libasan preloaded:
#   HDT_ORACLE_SANITIZE=1 ASAN_OPTIONS=detect_leaks=0 LD_PRELOAD=$(gcc -print-file-name=libasan.so) \
#       python -m pytest tests -m "not gpu" --deselect tests/test_abi.py
_SANITIZE = os.environ.get("HDT_ORACLE_SANITIZE", "") not in ("", "0")
_LIB = os.path.join(_HERE, "liboracle_san.so" if _SANITIZE else "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (fp64, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        flags = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                 "-fno-sanitize-recover=undefined"] if _SANITIZE else ["-O2"]
        cmd = ["gcc", *flags, "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i32p = ctypes.POINTER(ctypes.c_int32)
        i64p = ctypes.POINTER(ctypes.c_int64)
        u32p = ctypes.POINTER(ctypes.c_uint32)
        f64p = ctypes.POINTER(ctypes.c_double)
        i64 = ctypes.c_int64
        lib.oracle_allowed.argtypes = [i32p, i32p, i64, i64]
        lib.oracle_allowed.restype = ctypes.c_int
        lib.oracle_allowed_edges.argtypes = [i32p, i32p, i64, i64, ctypes.c_int]
        lib.oracle_allowed_edges.restype = ctypes.c_int
        lib.oracle_set_edges.argtypes = [ctypes.c_int]
        lib.oracle_set_edges.restype = None
        lib.oracle_get_edges.argtypes = []
        lib.oracle_get_edges.restype = ctypes.c_int
        lib.oracle_mask.argtypes = [i32p, i32p, i64, ctypes.POINTER(ctypes.c_uint8)]
        lib.oracle_mask.restype = None
        lib.oracle_row_counts.argtypes = [i32p, i32p, i64, i64p]
        lib.oracle_row_counts.restype = i64
        lib.oracle_row_lists.argtypes = [i32p, i32p, i64, i64p, i32p]
        lib.oracle_row_lists.restype = None
        lib.oracle_attn_fwd.argtypes = [f64p, f64p, f64p, i64, i64, i64, ctypes.c_double, i64p, i32p, f64p, f64p]
        lib.oracle_attn_fwd.restype = None
        lib.oracle_attn_bwd.argtypes = [f64p, f64p, f64p, f64p, i64, i64, i64, ctypes.c_double, i64p, i32p,
                                        f64p, f64p, f64p]
        lib.oracle_attn_bwd.restype = None
        lib.oracle_kperm.argtypes = [i32p, i64, i32p]
        lib.oracle_kperm.restype = None
        lib.oracle_block_scan.argtypes = [i32p, i32p, i32p, i64, i64, i64, i32p, u32p]
        lib.oracle_block_scan.restype = None
        lib.oracle_block_bitmaps.argtypes = [i32p, i32p, i32p, i64, i64, i64, i64, i32p, i32p, u32p]
        lib.oracle_block_bitmaps.restype = None
        lib.oracle_keylist_counts.argtypes = [i32p, i32p, i64, i64, i32p]
        lib.oracle_keylist_counts.restype = None
        lib.oracle_keylist_fill.argtypes = [i32p, i32p, i32p, i64, i64, i64, i64p, i32p, u32p, i32p]
        lib.oracle_keylist_fill.restype = None
        lib.oracle_index_vectors.argtypes = [i32p, i32p, i64, i64, i32p]
        lib.oracle_index_vectors.restype = None
        lib.oracle_hpe.argtypes = [i32p, i64, i64, i64, f64p]
        lib.oracle_hpe.restype = None
        lib.oracle_num_threads.argtypes = []
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


EDGE_UP, EDGE_SIBLING, EDGE_DOWN, EDGE_ALL = 1, 2, 4, 7


class edges:
    """``with oracle.edges(EDGE_SIBLING | EDGE_DOWN): ...`` evaluates every oracle function inside the
    block under a thinned mask (Sec. 4.1: the ListOps variants); the full pattern is restored after."""

    def __init__(self, kinds: int):
        self.kinds = int(kinds)

    def __enter__(self):
        lib = _load()
        self.saved = lib.oracle_get_edges()
        lib.oracle_set_edges(self.kinds)
        return self

    def __exit__(self, *exc):
        _load().oracle_set_edges(self.saved)
        return False


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def allowed(level, parent, i: int, j: int) -> bool:
    level, parent = _i32(level), _i32(parent)
    return bool(_load().oracle_allowed(_p(level, ctypes.c_int32), _p(parent, ctypes.c_int32), i, j))


def mask(level, parent) -> np.ndarray:
    """Dense 0/1 mask [n][n] of one sample."""
    level, parent = _i32(level), _i32(parent)
    n = level.shape[0]
    M = np.zeros((n, n), dtype=np.uint8)
    _load().oracle_mask(_p(level, ctypes.c_int32), _p(parent, ctypes.c_int32), n, _p(M, ctypes.c_uint8))
    return M


def row_lists(level, parent):
    """(rowptr int64[n+1], cols int32[nnz]) of one sample's mask, by pairwise enumeration."""
    level, parent = _i32(level), _i32(parent)
    n = level.shape[0]
    counts = np.zeros(n, dtype=np.int64)
    lib = _load()
    total = lib.oracle_row_counts(_p(level, ctypes.c_int32), _p(parent, ctypes.c_int32), n, _p(counts, ctypes.c_int64))
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    assert rowptr[-1] == total
    cols = np.zeros(max(int(total), 1), dtype=np.int32)
    lib.oracle_row_lists(_p(level, ctypes.c_int32), _p(parent, ctypes.c_int32), n, _p(rowptr, ctypes.c_int64),
                         _p(cols, ctypes.c_int32))
    return rowptr, cols[: int(total)]


def attn_fwd(q, k, v, level, parent, scale: float):
    """Masked softmax attention by definition.  q,k,v: [B][H][N][d] (any float dtype, widened to
    fp64); level,parent: [B][N].  Returns (o fp64 [B][H][N][d], lse fp64 [B][H][N])."""
    q = np.ascontiguousarray(q, dtype=np.float64)
    k = np.ascontiguousarray(k, dtype=np.float64)
    v = np.ascontiguousarray(v, dtype=np.float64)
    B, H, N, d = q.shape
    o = np.zeros_like(q)
    lse = np.zeros((B, H, N), dtype=np.float64)
    lib = _load()
    for b in range(B):
        rowptr, cols = row_lists(level[b], parent[b])
        cols_c = np.ascontiguousarray(cols if cols.size else np.zeros(1, np.int32))
        lib.oracle_attn_fwd(_p(q[b], ctypes.c_double), _p(k[b], ctypes.c_double), _p(v[b], ctypes.c_double),
                            H, N, d, float(scale), _p(rowptr, ctypes.c_int64), _p(cols_c, ctypes.c_int32),
                            _p(o[b], ctypes.c_double), _p(lse[b], ctypes.c_double))
    return o, lse


def attn_bwd(q, k, v, d_o, level, parent, scale: float):
    """Gradients (dq, dk, dv), fp64 [B][H][N][d], of sum(O * dO) w.r.t. q, k, v."""
    q = np.ascontiguousarray(q, dtype=np.float64)
    k = np.ascontiguousarray(k, dtype=np.float64)
    v = np.ascontiguousarray(v, dtype=np.float64)
    d_o = np.ascontiguousarray(d_o, dtype=np.float64)
    B, H, N, d = q.shape
    dq, dk, dv = np.zeros_like(q), np.zeros_like(q), np.zeros_like(q)
    lib = _load()
    for b in range(B):
        rowptr, cols = row_lists(level[b], parent[b])
        cols_c = np.ascontiguousarray(cols if cols.size else np.zeros(1, np.int32))
        lib.oracle_attn_bwd(_p(q[b], ctypes.c_double), _p(k[b], ctypes.c_double), _p(v[b], ctypes.c_double),
                            _p(d_o[b], ctypes.c_double), H, N, d, float(scale), _p(rowptr, ctypes.c_int64),
                            _p(cols_c, ctypes.c_int32), _p(dq[b], ctypes.c_double), _p(dk[b], ctypes.c_double),
                            _p(dv[b], ctypes.c_double))
    return dq, dk, dv


def kperm(level) -> np.ndarray:
    """Sorted slot -> document position, keys ordered by level, ties in document order, pads last."""
    level = _i32(level)
    n = level.shape[0]
    out = np.zeros(max(n, 1), dtype=np.int32)
    _load().oracle_kperm(_p(level, ctypes.c_int32), n, _p(out, ctypes.c_int32))
    return out[:n]


@dataclass
class BlockSchedule:
    """Surviving blocks of one sample.  q_* lists blocks by query-block row (columns ascending);
    k_* is the exact transpose (rows ascending).  ``sub`` packs, for the 32x32 sub-blocks of a
    block (sub-block (r, c) -> bit r*(bn/32)+c): bits 0..15 = holds an allowed pair, bits 16..31 =
    every pair allowed.  ``full`` = every one of the bm*bn pairs is allowed.  ``bits`` is the
    row-major bitmap, uint32 [n_blocks][bm][bn/32]."""
    bm: int
    bn: int
    kperm: np.ndarray
    q_rowptr: np.ndarray
    q_cols: np.ndarray
    q_full: np.ndarray
    q_sub: np.ndarray
    bits: np.ndarray
    k_colptr: np.ndarray
    k_rows: np.ndarray
    k_tile: np.ndarray  # index into the q-ordered block list of each transposed entry
    nnz: int
    q_keys: np.ndarray = None  # int32 [n_blocks][bn]: document position behind every key slot, -1 for pads / past n


def block_schedule(level, parent, bm: int, bn: int, use_sort: bool = True, force_dense: bool = False) -> BlockSchedule:
    """Brute-force block schedule of one sample (App. A.1, Alg. 1: sort, partition, skip empty)."""
    level, parent = _i32(level), _i32(parent)
    n = level.shape[0]
    assert bm % 32 == 0 and bn % 32 == 0
    kp = kperm(level) if use_sort else np.arange(n, dtype=np.int32)
    tr, tc = -(-n // bm), -(-n // bn)
    count = np.zeros(max(tr * tc, 1), dtype=np.int32)
    lib = _load()
    kp_c = np.ascontiguousarray(kp if n else np.zeros(1, np.int32))
    if n:
        lib.oracle_block_scan(_p(level, ctypes.c_int32), _p(parent, ctypes.c_int32), _p(kp_c, ctypes.c_int32),
                              n, bm, bn, _p(count, ctypes.c_int32), None)
    count = count[: tr * tc].reshape(tr, tc)
    alive = np.ones_like(count, dtype=bool) if force_dense else count > 0
    bi, bj = np.nonzero(alive)  # row-major: rows ascending, columns ascending inside a row
    bi = bi.astype(np.int32)
    bj = bj.astype(np.int32)
    nb = bi.shape[0]
    wpr = bn // 32
    bits = np.zeros((max(nb, 1), bm, wpr), dtype=np.uint32)
    if nb:
        lib.oracle_block_bitmaps(_p(level, ctypes.c_int32), _p(parent, ctypes.c_int32), _p(kp_c, ctypes.c_int32),
                                 n, bm, bn, nb, _p(np.ascontiguousarray(bi), ctypes.c_int32),
                                 _p(np.ascontiguousarray(bj), ctypes.c_int32), _p(bits, ctypes.c_uint32))
    bits = bits[:nb]
    q_rowptr = np.zeros(tr + 1, dtype=np.int32)
    np.cumsum(alive.sum(axis=1), out=q_rowptr[1:])
    q_full = (count[bi, bj] == bm * bn).astype(np.uint8) if nb else np.zeros(0, np.uint8)
    # 32x32 sub-block summaries from the bitmaps
    q_sub = np.zeros(nb, dtype=np.uint32)
    for r in range(bm // 32):
        for c in range(wpr):
            words = bits[:, r * 32:(r + 1) * 32, c] if nb else np.zeros((0, 32), np.uint32)
            any_ = (words != 0).any(axis=1)
            all_ = (words == 0xFFFFFFFF).all(axis=1)
            q_sub |= (any_.astype(np.uint32) << np.uint32(r * wpr + c))
            q_sub |= (all_.astype(np.uint32) << np.uint32(16 + r * wpr + c))
    # transpose: by column, rows ascending
    order = np.lexsort((bi, bj)) if nb else np.zeros(0, np.int64)
    k_rows = bi[order].astype(np.int32)
    k_colptr = np.zeros(tc + 1, dtype=np.int32)
    np.cumsum(alive.sum(axis=0), out=k_colptr[1:])
    # the positions behind the key slots of every block (pads and slots past n: -1)
    kp_pad = np.full(tc * bn, -1, dtype=np.int32)
    kp_pad[:n] = np.where(level[kp] >= 0, kp, -1) if n else kp
    q_keys = kp_pad.reshape(tc, bn)[bj] if nb else np.zeros((0, bn), np.int32)
    return BlockSchedule(bm=bm, bn=bn, kperm=kp, q_rowptr=q_rowptr, q_cols=bj, q_full=q_full, q_sub=q_sub,
                         bits=bits, k_colptr=k_colptr, k_rows=k_rows, k_tile=order.astype(np.int32),
                         nnz=int(count.sum()), q_keys=q_keys)


def _sub_summary(bits: np.ndarray, bm: int, bn: int) -> np.ndarray:
    """Per entry: bit r*(bn/32)+c set iff 32x32 sub-block (r, c) of the bitmap holds a set bit; bit
    16 + r*(bn/32)+c iff all of its bits are set."""
    nb, wpr = bits.shape[0], bn // 32
    sub = np.zeros(nb, dtype=np.uint32)
    for r in range(bm // 32):
        for c in range(wpr):
            words = bits[:, r * 32:(r + 1) * 32, c] if nb else np.zeros((0, 32), np.uint32)
            sub |= ((words != 0).any(axis=1).astype(np.uint32) << np.uint32(r * wpr + c))
            sub |= ((words == 0xFFFFFFFF).all(axis=1).astype(np.uint32) << np.uint32(16 + r * wpr + c))
    return sub


@dataclass
class KeyListSchedule:
    """Per-query-block key lists of one sample (see ``oracle_keylist_fill``): entries
    [q_rowptr[I], q_rowptr[I+1]) belong to query block I; entry e holds the keys ``q_keys[e]``
    (document positions in key order, -1 past the end of the block's list) and the bitmap
    ``bits[e]`` (uint32 [bm][ceil(bn/32)], bit c%32 of word c/32 <=> row r may attend to key c).
    ``q_sub`` as in BlockSchedule (only when bm and bn are multiples of 32)."""
    bm: int
    bn: int
    kperm: np.ndarray
    q_rowptr: np.ndarray
    q_keys: np.ndarray
    bits: np.ndarray
    pairs: np.ndarray
    q_sub: np.ndarray
    nnz: int


def keylist_schedule(level, parent, bm: int, bn: int, use_sort: bool = True) -> KeyListSchedule:
    """Brute-force key lists of every query block of one sample."""
    level, parent = _i32(level), _i32(parent)
    n = level.shape[0]
    kp = kperm(level) if use_sort else np.arange(n, dtype=np.int32)
    tr, wpr = -(-n // bm), -(-bn // 32)
    lib = _load()
    ucount = np.zeros(max(tr, 1), dtype=np.int32)
    if n:
        lib.oracle_keylist_counts(_p(level, ctypes.c_int32), _p(parent, ctypes.c_int32), n, bm,
                                  _p(ucount, ctypes.c_int32))
    ucount = ucount[:tr]
    entry_ptr = np.zeros(tr + 1, dtype=np.int64)
    np.cumsum(-(-ucount.astype(np.int64) // bn), out=entry_ptr[1:])
    E = int(entry_ptr[-1])
    keys = np.zeros((max(E, 1), bn), dtype=np.int32)
    bits = np.zeros((max(E, 1), bm, wpr), dtype=np.uint32)
    pairs = np.zeros(max(E, 1), dtype=np.int32)
    if n:
        kp_c = np.ascontiguousarray(kp)
        lib.oracle_keylist_fill(_p(level, ctypes.c_int32), _p(parent, ctypes.c_int32), _p(kp_c, ctypes.c_int32),
                                n, bm, bn, _p(entry_ptr, ctypes.c_int64), _p(keys, ctypes.c_int32),
                                _p(bits, ctypes.c_uint32), _p(pairs, ctypes.c_int32))
    keys, bits, pairs = keys[:E], bits[:E], pairs[:E]
    q_sub = _sub_summary(bits, bm, bn) if (bm % 32 == 0 and bn % 32 == 0) else np.zeros(E, np.uint32)
    return KeyListSchedule(bm=bm, bn=bn, kperm=kp, q_rowptr=entry_ptr.astype(np.int32), q_keys=keys, bits=bits,
                           pairs=pairs, q_sub=q_sub, nnz=int(pairs.sum()))


def index_vectors(level, parent, n_levels: int) -> np.ndarray:
    """int32 [n][n_levels]: the index vector p = (p^1 .. p^L) of every position of one sample."""
    level, parent = _i32(level), _i32(parent)
    n = level.shape[0]
    p = np.zeros((max(n, 1), n_levels), dtype=np.int32)
    if n:
        _load().oracle_index_vectors(_p(level, ctypes.c_int32), _p(parent, ctypes.c_int32), n, n_levels,
                                     _p(p, ctypes.c_int32))
    return p[:n]


def hpe(p, d_model: int) -> np.ndarray:
    """fp64 [n][d_model]: the hierarchical positional encoding of index vectors p [n][L]."""
    p = np.ascontiguousarray(p, dtype=np.int32)
    n, L = p.shape
    out = np.zeros((max(n, 1), d_model), dtype=np.float64)
    if n:
        _load().oracle_hpe(_p(p, ctypes.c_int32), n, L, d_model, _p(out, ctypes.c_double))
    return out[:n]


# ---------------------------------------------------------------------------------------------------
# Decoder cross-attention over a subset of the encoder's positions (Sec. 4.2, FacetSum study: the decoder
# attends only to the [SEC] anchors, or additionally to the [SENT] anchors, or additionally to the regular
# tokens).  The subset is the set of non-pad encoder positions whose level is in a given set of levels
# (bit l of ``level_mask`` <=> level l is visible); every decoder row attends to all of it.  Plain numpy in
# fp64: the definition (softmax over the visible positions, then the weighted sum of their values), heads and
# rows at once through einsum.

def cross_select(level_enc, level_mask: int) -> np.ndarray:
    """Visible encoder positions of one sample, in document order."""
    lv = _i32(level_enc)
    vis = np.array([l >= 0 and l < 32 and ((level_mask >> int(l)) & 1) == 1 for l in lv], dtype=bool)
    return np.flatnonzero(vis).astype(np.int32)


def cross_attn_fwd(q, k, v, level_enc, level_mask: int, scale: float):
    """q [B][H][n_dec][d], k, v [B][H][n_enc][d], level_enc [B][n_enc] -> (o [B][H][n_dec][d], lse [B][H][n_dec]).
    A sample without visible positions gives o = 0, lse = -inf."""
    q, k, v = (np.asarray(x, dtype=np.float64) for x in (q, k, v))
    B, H, nd, d = q.shape
    o = np.zeros((B, H, nd, d))
    lse = np.full((B, H, nd), -np.inf)
    for b in range(B):
        sel = cross_select(level_enc[b], level_mask)
        if sel.size == 0:
            continue
        s = scale * np.einsum("hic,hjc->hij", q[b], k[b][:, sel])
        m = s.max(axis=-1, keepdims=True)
        e = np.exp(s - m)
        l = e.sum(axis=-1, keepdims=True)
        lse[b] = (m + np.log(l))[..., 0]
        o[b] = np.einsum("hij,hjc->hic", e / l, v[b][:, sel])
    return o, lse


def cross_attn_bwd(q, k, v, d_o, level_enc, level_mask: int, scale: float):
    """Gradients of cross_attn_fwd's o with respect to q, k, v given d_o (rows of k, v that are not visible
    get zero)."""
    q, k, v, d_o = (np.asarray(x, dtype=np.float64) for x in (q, k, v, d_o))
    B = q.shape[0]
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    for b in range(B):
        sel = cross_select(level_enc[b], level_mask)
        if sel.size == 0:
            continue
        ks, vs = k[b][:, sel], v[b][:, sel]
        s = scale * np.einsum("hic,hjc->hij", q[b], ks)
        s -= s.max(axis=-1, keepdims=True)
        p = np.exp(s)
        p /= p.sum(axis=-1, keepdims=True)
        o = np.einsum("hij,hjc->hic", p, vs)
        big_d = (d_o[b] * o).sum(axis=-1, keepdims=True)       # D_i = sum_c dO_ic O_ic
        dp = np.einsum("hic,hjc->hij", d_o[b], vs)
        ds = p * (dp - big_d)
        dq[b] = scale * np.einsum("hij,hjc->hic", ds, ks)
        dk[b][:, sel] = scale * np.einsum("hij,hic->hjc", ds, q[b])
        dv[b][:, sel] = np.einsum("hij,hic->hjc", p, d_o[b])
    return dq, dk, dv


def _rect_schedule(row_ok: np.ndarray, keys: np.ndarray, bm: int, bn: int, per_tile_has_rows: bool) -> KeyListSchedule:
    """Schedule of a mask that is a rectangle: row r (of len(row_ok) rows, tiled by bm) may attend to every
    key of ``keys`` iff row_ok[r].  Every row tile gets the same list (all keys, bn per entry, the last entry
    filled with -1); with ``per_tile_has_rows`` a tile without any allowed row gets no entries."""
    n_rows, wpr = row_ok.shape[0], -(-bn // 32)
    tr = -(-n_rows // bm)
    n_ent = -(-keys.shape[0] // bn)
    rowptr = np.zeros(tr + 1, dtype=np.int32)
    q_keys, bits, pairs = [], [], []
    for I in range(tr):
        ok = np.zeros(bm, dtype=bool)
        seg = row_ok[I * bm:(I + 1) * bm]
        ok[:seg.shape[0]] = seg
        if not (per_tile_has_rows and not ok.any()):
            for e in range(n_ent):
                kk = np.full(bn, -1, dtype=np.int32)
                chunk = keys[e * bn:(e + 1) * bn]
                kk[:chunk.shape[0]] = chunk
                w = np.zeros((bm, wpr), dtype=np.uint32)
                for r in range(bm):
                    if ok[r]:
                        for c in range(chunk.shape[0]):
                            w[r, c >> 5] |= np.uint32(1) << np.uint32(c & 31)
                q_keys.append(kk)
                bits.append(w)
                pairs.append(int(ok.sum()) * chunk.shape[0])
        rowptr[I + 1] = len(q_keys)
    E = len(q_keys)
    q_keys = np.array(q_keys, dtype=np.int32).reshape(E, bn)
    bits = np.array(bits, dtype=np.uint32).reshape(E, bm, wpr)
    pairs = np.array(pairs, dtype=np.int32).reshape(E)
    q_sub = _sub_summary(bits, bm, bn) if (bm % 32 == 0 and bn % 32 == 0) else np.zeros(E, np.uint32)
    return KeyListSchedule(bm=bm, bn=bn, kperm=np.zeros(0, np.int32), q_rowptr=rowptr, q_keys=q_keys, bits=bits,
                           pairs=pairs, q_sub=q_sub, nnz=int(pairs.sum()))


def cross_schedule(level_enc, n_dec: int, level_mask: int, bm: int, bn: int):
    """(forward schedule, transposed schedule) of one sample's cross-attention mask.  Forward: rows are the
    decoder positions, every row tile lists the visible encoder positions in document order.  Transposed
    (for dK, dV): rows are the encoder positions (allowed iff visible), a tile with a visible row lists all
    decoder positions."""
    sel = cross_select(level_enc, level_mask)
    n_enc = _i32(level_enc).shape[0]
    fwd = _rect_schedule(np.ones(n_dec, dtype=bool), sel, bm, bn, per_tile_has_rows=False)
    vis = np.zeros(n_enc, dtype=bool)
    vis[sel] = True
    tr_ = _rect_schedule(vis, np.arange(n_dec, dtype=np.int32), bm, bn, per_tile_has_rows=True)
    return fwd, tr_


def parents_from_levels(level) -> np.ndarray:
    """Parent index of every position of a document laid out as Sec. 3.2 describes it: anchors in front of what
    they summarise ([DOC] first, a [SEC] at the start of its section, a [SENT] at the start of its sentence),
    i.e. in pre-order.  The parent of a position of level l > 0 is then the nearest earlier position of level
    l - 1; level 0, pads and positions without such a predecessor have none (-1).  Plain loop."""
    level = _i32(level)
    parent = np.full(level.shape[0], -1, dtype=np.int32)
    for i in range(level.shape[0]):
        if level[i] > 0:
            for j in range(i - 1, -1, -1):
                if level[j] == level[i] - 1:
                    parent[i] = j
                    break
    return parent
