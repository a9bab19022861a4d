"""Reference formulas used to pin the oracle; written independently of it (numpy only)."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_golden_mask(name):
    level = parent = kperm = None
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("level"):
                level = np.array(line.split()[1:], dtype=np.int32)
            elif line.startswith("parent"):
                parent = np.array(line.split()[1:], dtype=np.int32)
            elif line.startswith("kperm"):
                kperm = np.array(line.split()[1:], dtype=np.int32)
            else:
                rows.append([int(c) for c in line])
    return level, parent, kperm, np.array(rows, dtype=np.uint8)


def index_vectors(sections, n_pos):
    """Index vectors p = (p1, p2, p3) of a 3-level document laid out in pre-order with anchors
    prepended (paper Fig. 3): 1-based, an anchor carries 0 at every level below its own.
    Returns int array [n_pos][3] and a validity flag per position (pads are invalid)."""
    p = np.zeros((n_pos, 3), dtype=np.int64)
    valid = np.zeros(n_pos, dtype=bool)
    pos = 0
    valid[pos] = True  # [DOC] = (0, 0, 0)
    pos += 1
    for k, sec in enumerate(sections, start=1):
        p[pos] = (k, 0, 0)
        valid[pos] = True
        pos += 1
        for m, length in enumerate(sec, start=1):
            p[pos] = (k, m, 0)
            valid[pos] = True
            pos += 1
            for t in range(1, length + 1):
                p[pos] = (k, m, t)
                valid[pos] = True
                pos += 1
    return p, valid


def mask_from_equations(sections, n_pos):
    """M = M_DOC or M_SEC or M_SENT, the three equations of paper Sec. 3.2, on index vectors."""
    p, valid = index_vectors(sections, n_pos)
    p1, p2, p3 = p[:, 0], p[:, 1], p[:, 2]
    m_doc = (p2[:, None] == 0) & (p2[None, :] == 0)
    m_sec = (p3[:, None] == 0) & (p3[None, :] == 0) & (p1[:, None] == p1[None, :])
    m_sent = (p1[:, None] == p1[None, :]) & (p2[:, None] == p2[None, :])
    M = m_doc | m_sec | m_sent
    M &= valid[:, None] & valid[None, :]
    return M.astype(np.uint8)


def dense_masked_attention(q, k, v, M, scale):
    """Textbook softmax attention (paper Eq. 1 with the -inf masking of Sec. 3.2) for one head in
    fp64 with a dense mask; rows without any allowed key give o = 0, lse = -inf."""
    a = scale * (q.astype(np.float64) @ k.astype(np.float64).T)
    a = np.where(M.astype(bool), a, -np.inf)
    m = a.max(axis=1, keepdims=True)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    e = np.exp(a - m_safe)
    z = e.sum(axis=1, keepdims=True)
    with np.errstate(divide="ignore", invalid="ignore"):
        s = np.where(z > 0, e / np.where(z > 0, z, 1.0), 0.0)
        lse = np.where(z[:, 0] > 0, m_safe[:, 0] + np.log(np.where(z[:, 0] > 0, z[:, 0], 1.0)), -np.inf)
    return s @ v.astype(np.float64), lse, s
