"""Seeded synthetic inputs: document hierarchies and Q/K/V/dO tensors.

This module only *draws inputs*.  It holds none of the method's arithmetic (no
mask rule, no key ordering, no tiling, no softmax), so that both the HIP path
and the CPU oracle can be fed from it without sharing any logic.

A document is the pre-order listing of a tree whose inner nodes are anchor
positions: one [DOC] anchor, one [SEC] anchor in front of every section and one
[SENT] anchor in front of every sentence (paper Sec. 3.2, "Hierarchical
Document Transformer": anchors are prepended to the element they stand for).
Each position carries

    level   0 = [DOC], 1 = [SEC], 2 = [SENT], 3 = regular token, -1 = pad
    parent  index (inside the same sample) of the enclosing anchor,
            -1 for the root and for pads

The five workload recipes below follow the shapes and distributions the
benchmark contract names (encoder-sized 4096, long-document 8192 with one
skewed 600-token sentence, training step at 8192, stress 32768); they stand in
for the real corpora the paper measured on, which are not available here.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

LEVEL_DOC = 0
LEVEL_SEC = 1
LEVEL_SENT = 2
LEVEL_TOKEN = 3
LEVEL_PAD = -1

SEED_BASE = 24070833 * 10


def sample_seed(config: int, sample: int) -> int:
    return SEED_BASE + config * 100 + sample


def document_from_sections(sections: Sequence[Sequence[int]], n_pos: int):
    """Lay out ``sections`` (a list of sections, each a list of sentence lengths in
    regular tokens) in pre-order with anchors prepended and pad to ``n_pos``.

    Returns (level[n_pos], parent[n_pos]) as int32 arrays."""
    level = np.full(n_pos, LEVEL_PAD, dtype=np.int32)
    parent = np.full(n_pos, -1, dtype=np.int32)
    need = 1 + sum(1 + sum(1 + int(l) for l in sec) for sec in sections)
    if need > n_pos:
        raise ValueError(f"document needs {need} positions, only {n_pos} available")
    pos = 0
    doc = pos
    level[pos] = LEVEL_DOC
    pos += 1
    for sec in sections:
        sec_pos = pos
        level[pos] = LEVEL_SEC
        parent[pos] = doc
        pos += 1
        for length in sec:
            sent_pos = pos
            level[pos] = LEVEL_SENT
            parent[pos] = sec_pos
            pos += 1
            length = int(length)
            level[pos:pos + length] = LEVEL_TOKEN
            parent[pos:pos + length] = sent_pos
            pos += length
    return level, parent


def tree_document(children_counts_by_depth, rng: np.random.Generator, n_pos: Optional[int] = None,
                  max_nodes: int = 4096):
    """A generic pre-order tree of arbitrary depth for tests.

    ``children_counts_by_depth[d] = (lo, hi)`` is the inclusive range of the number of
    children drawn for a node at depth d; nodes at depth len(children_counts_by_depth)
    are leaves.  Level of a node = its depth."""
    levels: List[int] = []
    parents: List[int] = []

    def grow(depth: int, par: int):
        if len(levels) >= max_nodes:
            return
        me = len(levels)
        levels.append(depth)
        parents.append(par)
        if depth < len(children_counts_by_depth):
            lo, hi = children_counts_by_depth[depth]
            for _ in range(int(rng.integers(lo, hi + 1))):
                grow(depth + 1, me)

    grow(0, -1)
    n_real = len(levels)
    if n_pos is None:
        n_pos = n_real
    if n_real > n_pos:
        raise ValueError("tree larger than n_pos")
    level = np.full(n_pos, LEVEL_PAD, dtype=np.int32)
    parent = np.full(n_pos, -1, dtype=np.int32)
    level[:n_real] = np.asarray(levels, dtype=np.int32)
    parent[:n_real] = np.asarray(parents, dtype=np.int32)
    return level, parent


def listops_like_tree(rng: np.random.Generator, n_pos: int, max_depth: int = 20, max_nodes: Optional[int] = None):
    """A nested-list expression in the shape of the ListOps task (paper Sec. 4.1: operators with 2-5
    operands, nesting depth up to 20), written in pre-order: an operator position followed by its
    operands, each a leaf or another bracketed expression.  Only the SHAPE is drawn (which operand is
    nested, how many operands); no operator names, digits or task items are involved.
    level = nesting depth, parent = the enclosing operator.  Returns (level[n_pos], parent[n_pos])
    padded with pads; the tree holds at most ``max_nodes`` (default n_pos) positions."""
    cap = n_pos if max_nodes is None else min(max_nodes, n_pos)
    levels: List[int] = [0]
    parents: List[int] = [-1]
    # depth-first growth in pre-order; the stack holds (operator position, depth, operands still to write)
    stack = [(0, 0, int(rng.integers(2, 6)))]
    while stack and len(levels) < cap:
        op, depth, left = stack.pop()
        if left == 0:
            continue
        stack.append((op, depth, left - 1))
        me = len(levels)
        levels.append(depth + 1)
        parents.append(op)
        # a nested expression with a probability that keeps the expected size finite but reaches deep trees
        if depth + 1 < max_depth and rng.random() < 0.42:
            stack.append((me, depth + 1, int(rng.integers(2, 6))))
    level = np.full(n_pos, LEVEL_PAD, dtype=np.int32)
    parent = np.full(n_pos, -1, dtype=np.int32)
    level[:len(levels)] = levels
    parent[:len(parents)] = parents
    return level, parent


def _fill_sections(rng, n_pos, sent_per_sec, sent_len, forced=None):
    """Append sections sentence by sentence until the next piece does not fit.

    A sentence (anchor + tokens) is only appended when it fits entirely; a new
    section is only opened when its [SEC] anchor and its first sentence fit.  The
    first misfit ends the document.  ``forced`` = (section, sentence, length) overrides
    one drawn sentence length."""
    sections: List[List[int]] = []
    used = 1  # [DOC]
    while True:
        k = int(rng.integers(sent_per_sec[0], sent_per_sec[1] + 1))
        sec: List[int] = []
        opened = False
        stop = False
        for m in range(k):
            length = int(rng.integers(sent_len[0], sent_len[1] + 1))
            if forced is not None and forced[0] == len(sections) and forced[1] == m:
                length = forced[2]
            cost = 1 + length + (0 if opened else 1)
            if used + cost > n_pos:
                stop = True
                break
            used += cost
            opened = True
            sec.append(length)
        if sec:
            sections.append(sec)
        if stop:
            break
    return sections


def pseudo_section_document(rng: np.random.Generator, n_pos: int, sent_len=(10, 80), per_section: int = 32):
    """Unstructured text as the paper treats it (Sec. 4.2, SCROLLS): sentences grouped into
    pseudo-sections of a fixed number of sentences (32).  Sentence lengths are drawn uniform; the
    document is filled as by the other recipes (a sentence only if it fits entirely)."""
    sections = _fill_sections(rng, n_pos, (per_section, per_section), sent_len)
    level, parent = document_from_sections(sections, n_pos)
    return level, parent, sections


def _budgeted_sections(rng, n_pos, n_sections, sent_per_sec, sent_len):
    """Exactly ``n_sections`` sections under a running position budget: section s may grow
    until the document holds floor((s+1)*(n_pos-1)/n_sections) positions (at least one
    sentence each, shortened to fit if need be)."""
    sections: List[List[int]] = []
    used = 1
    for s in range(n_sections):
        budget = ((s + 1) * (n_pos - 1)) // n_sections + 1
        k = int(rng.integers(sent_per_sec[0], sent_per_sec[1] + 1))
        sec: List[int] = []
        used += 1  # [SEC]
        for m in range(k):
            length = int(rng.integers(sent_len[0], sent_len[1] + 1))
            if used + 1 + length > budget:
                if not sec:
                    length = max(1, min(length, budget - used - 1))
                    if used + 1 + length > budget:
                        raise ValueError("budget too small for one sentence")
                    sec.append(length)
                    used += 1 + length
                break
            sec.append(length)
            used += 1 + length
        sections.append(sec)
    return sections


@dataclass
class Workload:
    """One benchmark configuration: shapes plus the per-sample hierarchies."""
    name: str
    config: int
    batch: int
    heads: int
    head_dim: int
    n_pos: int
    dtype: str  # "bf16" or "f32"
    backward: bool
    level: np.ndarray = field(repr=False, default=None)   # int32 [B][N]
    parent: np.ndarray = field(repr=False, default=None)  # int32 [B][N]
    sections: list = field(repr=False, default=None)      # per sample: list of sections

    @property
    def softmax_scale(self) -> float:
        return 1.0 / float(np.sqrt(self.head_dim))

    @property
    def n_real(self) -> int:
        return int((self.level >= 0).sum())


_CONFIG_SHAPES = {
    1: dict(name="tiny-fwd-f32", batch=1, heads=1, head_dim=64, n_pos=512, dtype="f32", backward=False),
    2: dict(name="encoder-4096-fwd", batch=8, heads=12, head_dim=64, n_pos=4096, dtype="bf16", backward=False),
    3: dict(name="longdoc-8192-fwd", batch=4, heads=12, head_dim=64, n_pos=8192, dtype="bf16", backward=False),
    4: dict(name="train-8192-fwd-bwd", batch=4, heads=12, head_dim=64, n_pos=8192, dtype="bf16", backward=True),
    5: dict(name="stress-32768", batch=1, heads=16, head_dim=128, n_pos=32768, dtype="bf16", backward=True),
}


def make_workload(config: int, batch: Optional[int] = None, heads: Optional[int] = None) -> Workload:
    """Hierarchies for benchmark configuration ``config`` (1..5).  ``batch``/``heads`` may be
    reduced for tests; sample s of a reduced batch equals sample s of the full one."""
    if config not in _CONFIG_SHAPES:
        raise ValueError("config must be 1..5")
    shp = dict(_CONFIG_SHAPES[config])
    if batch is not None:
        shp["batch"] = batch
    if heads is not None:
        shp["heads"] = heads
    wl = Workload(config=config, **shp)
    levels, parents, secs = [], [], []
    hier_cfg = 3 if config == 4 else config  # config 4 reuses config 3's documents
    for s in range(wl.batch):
        rng = np.random.default_rng(sample_seed(hier_cfg, s))
        if config == 1:
            sections = [[int(rng.integers(5, 61)) for _ in range(4)] for _ in range(2)]
        elif config == 2:
            sections = _fill_sections(rng, wl.n_pos, (3, 30), (5, 60))
        elif config in (3, 4):
            forced = None
            if s == 0:
                # the skewed document: the middle sentence of its first section has 600 tokens
                probe = np.random.default_rng(sample_seed(hier_cfg, s))
                k0 = int(probe.integers(3, 31))
                forced = (0, k0 // 2, 600)
            sections = _fill_sections(rng, wl.n_pos, (3, 30), (10, 80), forced)
        else:
            sections = _budgeted_sections(rng, wl.n_pos, 64, (5, 40), (5, 60))
        lv, pr = document_from_sections(sections, wl.n_pos)
        levels.append(lv)
        parents.append(pr)
        secs.append(sections)
    wl.level = np.stack(levels)
    wl.parent = np.stack(parents)
    wl.sections = secs
    return wl


def make_qkv(batch: int, heads: int, n_pos: int, head_dim: int, seed: int, n_tensors: int = 3):
    """``n_tensors`` iid N(0,1) float32 arrays of shape [B][H][N][d] (Q, K, V and, when
    n_tensors == 4, dO)."""
    rng = np.random.default_rng(seed)
    return [rng.standard_normal((batch, heads, n_pos, head_dim), dtype=np.float32) for _ in range(n_tensors)]


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even) and return them as float32.
    Pure bit manipulation, so neither side depends on a device library for it."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    rounded = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return rounded.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16).reshape(x.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)
