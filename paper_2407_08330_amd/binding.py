"""ctypes binding of libhdt.so: argument marshalling only.  Every step of the method runs in the
HIP kernels behind the C ABI declared in ``include/hdt.h``; there is no fallback path, and a
missing library is an error."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libhdt.so")
_lib = None

HDT_BF16, HDT_F32 = 0, 1
HDT_EDGE_UP, HDT_EDGE_SIBLING, HDT_EDGE_DOWN, HDT_EDGE_ALL = 1, 2, 4, 7

EXPORTED_SYMBOLS = [
    "hdt_build_layout", "hdt_build_cross_layout", "hdt_layout_transposed", "hdt_layout_status", "hdt_layout_info", "hdt_layout_sample_info", "hdt_layout_export", "hdt_layout_destroy", "hdt_layout_destroy_completed",
    "hdt_attn_fwd", "hdt_attn_fwd_ws", "hdt_attn_fwd_workspace_bytes", "hdt_attn_bwd_workspace_bytes", "hdt_attn_bwd", "hdt_attn_bwd_no_alloc", "hdt_status_string", "hdt_last_error",
    "hdt_timing_enable", "hdt_timing_reset", "hdt_timing_read", "hdt_probe_mfma_bf16", "hdt_release_cached_memory",
    "hdt_parents_from_levels", "hdt_index_vectors_workspace_bytes", "hdt_index_vectors", "hdt_hpe_table", "hdt_hpe_add",
]


class HdtError(RuntimeError):
    def __init__(self, status: int, name: str, text: str):
        super().__init__(f"{name} ({status}): {text}")
        self.status = status
        self.name = name


class _Opts(ctypes.Structure):
    _fields_ = [("tile_m", ctypes.c_int32), ("tile_n", ctypes.c_int32), ("force_dense", ctypes.c_int32),
                ("no_sort", ctypes.c_int32), ("windowed", ctypes.c_int32), ("edges", ctypes.c_int32),
                ("deferred", ctypes.c_int32), ("reserved", ctypes.c_int32), ("capacity", ctypes.c_int64)]


class _Info(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_pos", ctypes.c_int32), ("tile_m", ctypes.c_int32),
                ("tile_n", ctypes.c_int32), ("q_tiles", ctypes.c_int32), ("k_tiles", ctypes.c_int32),
                ("windowed", ctypes.c_int32), ("edges", ctypes.c_int32), ("n_tiles", ctypes.c_int64),
                ("nnz", ctypes.c_int64), ("device_bytes", ctypes.c_int64), ("n_kv", ctypes.c_int32),
                ("cross", ctypes.c_int32), ("cross_level_mask", ctypes.c_uint32), ("compact_rows", ctypes.c_int32)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libhdt.so built in-tree (``python -m paper_2407_08330_amd.build`` or
    ``__graft_entry__.build()``).  Raises if it is missing: there is no other path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(f"{_LIB_PATH} not built; run __graft_entry__.build() first")
    # PyTorch-ROCm ships its own HIP runtime.  Import it first so that libhdt binds to that same
    # copy: two HIP runtimes in one process do not see each other's device state.
    import torch  # noqa: F401
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    lib.hdt_build_layout.argtypes = [vp, vp, i32, i32, ctypes.POINTER(_Opts), vp, ctypes.POINTER(vp)]
    lib.hdt_build_layout.restype = ctypes.c_int
    lib.hdt_build_cross_layout.argtypes = [vp, i32, i32, i32, ctypes.c_uint32, ctypes.POINTER(_Opts), vp, ctypes.POINTER(vp)]
    lib.hdt_build_cross_layout.restype = ctypes.c_int
    lib.hdt_layout_transposed.argtypes = [vp, ctypes.POINTER(vp)]
    lib.hdt_layout_transposed.restype = ctypes.c_int
    lib.hdt_layout_status.argtypes = [vp, ctypes.POINTER(i64)]
    lib.hdt_layout_status.restype = ctypes.c_int
    lib.hdt_layout_info.argtypes = [vp, ctypes.POINTER(_Info)]
    lib.hdt_layout_info.restype = ctypes.c_int
    lib.hdt_layout_sample_info.argtypes = [vp, i32, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    lib.hdt_layout_sample_info.restype = ctypes.c_int
    lib.hdt_layout_export.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64]
    lib.hdt_layout_export.restype = ctypes.c_int
    lib.hdt_layout_destroy.argtypes = [vp]
    lib.hdt_layout_destroy.restype = ctypes.c_int
    lib.hdt_layout_destroy_completed.argtypes = [vp]
    lib.hdt_layout_destroy_completed.restype = ctypes.c_int
    lib.hdt_attn_fwd.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, ctypes.c_int, f32, vp]
    lib.hdt_attn_fwd.restype = ctypes.c_int
    lib.hdt_attn_fwd_ws.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, ctypes.c_int, f32, vp, ctypes.c_size_t, vp]
    lib.hdt_attn_fwd_ws.restype = ctypes.c_int
    lib.hdt_attn_fwd_workspace_bytes.argtypes = [vp, i32, i32, ctypes.c_int]
    lib.hdt_attn_fwd_workspace_bytes.restype = ctypes.c_size_t
    lib.hdt_attn_bwd_workspace_bytes.argtypes = [vp, i32, i32, ctypes.c_int]
    lib.hdt_attn_bwd_workspace_bytes.restype = ctypes.c_size_t
    lib.hdt_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, ctypes.c_int, f32, vp,
                                 ctypes.c_size_t, vp]
    lib.hdt_attn_bwd.restype = ctypes.c_int
    lib.hdt_attn_bwd_no_alloc.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, ctypes.c_int, f32, vp]
    lib.hdt_attn_bwd_no_alloc.restype = ctypes.c_int
    lib.hdt_status_string.argtypes = [ctypes.c_int]
    lib.hdt_status_string.restype = ctypes.c_char_p
    lib.hdt_last_error.argtypes = []
    lib.hdt_last_error.restype = ctypes.c_char_p
    lib.hdt_timing_enable.argtypes = [i32]
    lib.hdt_timing_enable.restype = ctypes.c_int
    lib.hdt_timing_reset.argtypes = []
    lib.hdt_timing_reset.restype = ctypes.c_int
    lib.hdt_timing_read.argtypes = [ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(i64),
                                    ctypes.POINTER(ctypes.c_double), i32]
    lib.hdt_timing_read.restype = i32
    lib.hdt_probe_mfma_bf16.argtypes = [i32, i32, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.hdt_probe_mfma_bf16.restype = ctypes.c_int
    lib.hdt_release_cached_memory.argtypes = []
    lib.hdt_release_cached_memory.restype = ctypes.c_int
    lib.hdt_parents_from_levels.argtypes = [vp, i32, i32, vp, vp]
    lib.hdt_parents_from_levels.restype = ctypes.c_int
    lib.hdt_index_vectors_workspace_bytes.argtypes = [i32, i32]
    lib.hdt_index_vectors_workspace_bytes.restype = ctypes.c_size_t
    lib.hdt_index_vectors.argtypes = [vp, vp, i32, i32, i32, vp, vp, ctypes.c_size_t, vp]
    lib.hdt_index_vectors.restype = ctypes.c_int
    lib.hdt_hpe_table.argtypes = [vp, i32, i32, vp]
    lib.hdt_hpe_table.restype = ctypes.c_int
    lib.hdt_hpe_add.argtypes = [vp, i32, i32, i32, vp, i32, vp, i32, ctypes.c_int, vp]
    lib.hdt_hpe_add.restype = ctypes.c_int
    _lib = lib
    return lib


def _check(status: int):
    if status != 0:
        lib = load_library()
        raise HdtError(status, lib.hdt_status_string(status).decode(), lib.hdt_last_error().decode())


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def _scratch(nbytes: int, device, stream):
    """A temporary uint8 device tensor for kernels enqueued on ``stream``.  It is dropped by the caller while
    those kernels may still be queued, so it is allocated in that stream's context: torch's allocator hands a
    freed block out again in the order of the stream it was allocated on."""
    import torch
    if stream is None:
        return torch.empty(max(nbytes, 16), dtype=torch.uint8, device=device)
    with torch.cuda.stream(stream):
        return torch.empty(max(nbytes, 16), dtype=torch.uint8, device=device)


class Layout:
    """Owns an ``hdt_layout_t``."""

    def __init__(self, handle: int, batch: int, n_pos: int, n_kv: Optional[int] = None, owner=None):
        self._h = ctypes.c_void_p(handle)
        self.batch, self.n_pos = int(batch), int(n_pos)
        self.n_kv = int(n_pos if n_kv is None else n_kv)   # rows of the gathered tensors (cross-attention: encoder)
        self._owner = owner                                 # a borrowed handle keeps its owner alive

    def transposed(self) -> Optional["Layout"]:
        """The schedule of the transposed mask held for the backward pass (borrowed), or None."""
        h = ctypes.c_void_p(0)
        _check(load_library().hdt_layout_transposed(self._h, ctypes.byref(h)))
        return Layout(h.value, self.batch, self.n_kv, self.n_pos, owner=self) if h.value else None

    @property
    def handle(self):
        return self._h

    def status(self) -> int:
        """Outcome of a deferred build: waits for the build kernel's report, raises HdtError if the build failed
        (``entries_needed`` on the exception is what ``capacity`` must be at least); returns the list entries
        the schedule needs."""
        need = ctypes.c_int64(0)
        st = load_library().hdt_layout_status(self._h, ctypes.byref(need))
        if st != 0:
            lib = load_library()
            err = HdtError(st, lib.hdt_status_string(st).decode(), lib.hdt_last_error().decode())
            err.entries_needed = need.value
            raise err
        return need.value

    def info(self) -> dict:
        info = _Info()
        _check(load_library().hdt_layout_info(self._h, ctypes.byref(info)))
        return {f: getattr(info, f) for f, _ in _Info._fields_}

    def sample_info(self, sample: int):
        a, b = ctypes.c_int64(0), ctypes.c_int64(0)
        _check(load_library().hdt_layout_sample_info(self._h, sample, ctypes.byref(a), ctypes.byref(b)))
        return a.value, b.value

    def export(self, sample: int) -> dict:
        """Host copies of one sample's schedule (numpy arrays, shapes as in hdt_layout_export)."""
        inf = self.info()
        T, _ = self.sample_info(sample)
        n, tr, tc, bm, bn = inf["n_pos"], inf["q_tiles"], inf["k_tiles"], inf["tile_m"], inf["tile_n"]
        out = dict(
            q_rowptr=np.zeros(tr + 1, np.int32),
            q_cols=np.zeros(max(T, 1), np.int32), q_keys=np.zeros((max(T, 1), bn), np.int32),
            q_sub=np.zeros(max(T, 1), np.uint32), bits=np.zeros((max(T, 1), bm, bn // 32), np.uint32))
        if not inf["cross"]:  # a cross-attention layout has no key order
            out["kperm"] = np.zeros(max(n, 1), np.int32)
        if inf["windowed"]:  # only a windowed layout has a transpose by key window
            out.update(k_colptr=np.zeros(tc + 1, np.int32), k_rows=np.zeros(max(T, 1), np.int32),
                       k_tile=np.zeros(max(T, 1), np.int32))
        p = {k: ctypes.c_void_p(v.ctypes.data) for k, v in out.items()}
        _check(load_library().hdt_layout_export(self._h, sample, p.get("kperm"), p["q_rowptr"], p["q_cols"], p["q_keys"],
                                                p["q_sub"], p["bits"], p.get("k_colptr"), p.get("k_rows"),
                                                p.get("k_tile"), max(T, 1)))
        if "kperm" in out:
            out["kperm"] = out["kperm"][:n]
        for key in ("q_cols", "q_keys", "q_sub", "bits", "k_rows", "k_tile"):
            if key in out:
                out[key] = out[key][:T]
        return out

    def destroy(self, completed: bool = False):
        """hdt_layout_destroy: the layout's device buffers go to the library's cache, and the build that takes them
        later runs behind the calls that used the layout (no host wait; the calls may still be queued).
        ``completed=True`` (hdt_layout_destroy_completed): the caller has waited for all of them already."""
        if self._owner is None and self._h is not None and self._h.value:
            lib = load_library()
            _check((lib.hdt_layout_destroy_completed if completed else lib.hdt_layout_destroy)(self._h))
        self._h = None
        self._owner = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def hdt_build_layout(level, parent, tile_m: int = 0, tile_n: int = 0, force_dense: bool = False,
                     no_sort: bool = False, windowed: bool = False, edges: int = 0, deferred: bool = False,
                     capacity: int = 0, stream=None) -> Layout:
    """level, parent: int32 device tensors [batch][n_pos].  ``edges``: OR of HDT_EDGE_* (0 = all).
    ``deferred``: only enqueue the build (see hdt_build_layout in include/hdt.h); ``capacity``: list entries
    the layout has room for (0 = the library chooses)."""
    import torch
    if level.dtype != torch.int32 or parent.dtype != torch.int32:
        raise TypeError("level and parent must be int32")
    if level.dim() != 2 or level.shape != parent.shape:
        raise ValueError("level and parent must both be [batch][n_pos]")
    if not (level.is_cuda and parent.is_cuda and level.is_contiguous() and parent.is_contiguous()):
        raise ValueError("level and parent must be contiguous device tensors")
    opts = _Opts(tile_m, tile_n, int(force_dense), int(no_sort), int(windowed), int(edges), int(deferred), 0,
                 int(capacity))
    h = ctypes.c_void_p(0)
    B, N = level.shape
    _check(load_library().hdt_build_layout(_ptr(level) if B * N else None, _ptr(parent) if B * N else None, B, N,
                                           ctypes.byref(opts), _stream_ptr(stream), ctypes.byref(h)))
    return Layout(h.value, B, N)


def hdt_build_cross_layout(level_enc, n_dec: int, level_mask: int, tile_m: int = 0, tile_n: int = 0,
                           stream=None) -> Layout:
    """level_enc: int32 device tensor [batch][n_enc]; decoder rows attend to the encoder positions whose
    level has its bit set in ``level_mask``.  The layout takes q, o of n_dec rows and k, v of n_enc rows."""
    import torch
    if level_enc.dtype != torch.int32 or level_enc.dim() != 2:
        raise TypeError("level_enc must be int32 [batch][n_enc]")
    if not (level_enc.is_cuda and level_enc.is_contiguous()):
        raise ValueError("level_enc must be a contiguous device tensor")
    opts = _Opts(tile_m, tile_n, 0, 0, 0, 0, 0, 0, 0)
    h = ctypes.c_void_p(0)
    B, n_enc = level_enc.shape
    _check(load_library().hdt_build_cross_layout(_ptr(level_enc) if B * n_enc else None, B, n_enc, int(n_dec),
                                                 int(level_mask), ctypes.byref(opts), _stream_ptr(stream),
                                                 ctypes.byref(h)))
    return Layout(h.value, B, int(n_dec), n_enc)


def _dtype_code(t):
    import torch
    if t.dtype == torch.bfloat16:
        return HDT_BF16
    if t.dtype == torch.float32:
        return HDT_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _check_tensors(ts, shape=None):
    for t in ts:
        if not (t.is_cuda and t.is_contiguous()):
            raise ValueError("tensors must be contiguous device tensors")
        if shape is not None and tuple(t.shape) != tuple(shape):
            raise ValueError(f"tensor shape {tuple(t.shape)} != {tuple(shape)}")


def hdt_attn_fwd_workspace_bytes(layout: Layout, heads: int, head_dim: int, dtype_code: int) -> int:
    return int(load_library().hdt_attn_fwd_workspace_bytes(layout.handle, heads, head_dim, dtype_code))


def hdt_attn_fwd(layout: Layout, q, k, v, softmax_scale: float, o=None, lse=None, workspace=None, stream=None):
    """q: [batch][heads][n_pos][head_dim], k, v: [batch][heads][n_kv][head_dim] device tensors (bf16 or fp32;
    n_kv = n_pos unless the layout is a cross-attention layout).  ``workspace``: a uint8 device tensor for
    hdt_attn_fwd_ws (long key lists of a cross-attention layout cut into pieces).  Returns (o, lse)."""
    import torch
    B, H, N, D = q.shape
    _check_tensors((q,), q.shape)
    _check_tensors((k, v), (B, H, layout.n_kv, D))
    if (B, N) != (layout.batch, layout.n_pos) or k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("tensor shapes or dtypes do not match the layout")
    if o is None:
        o = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
    if workspace is not None:
        _check(load_library().hdt_attn_fwd_ws(layout.handle, _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), H, D,
                                              _dtype_code(q), float(softmax_scale), _ptr(workspace),
                                              workspace.numel() * workspace.element_size(), _stream_ptr(stream)))
        return o, lse
    _check(load_library().hdt_attn_fwd(layout.handle, _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), H, D,
                                       _dtype_code(q), float(softmax_scale), _stream_ptr(stream)))
    return o, lse


def hdt_attn_bwd_workspace_bytes(layout: Layout, heads: int, head_dim: int, dtype_code: int) -> int:
    return int(load_library().hdt_attn_bwd_workspace_bytes(layout.handle, heads, head_dim, dtype_code))


def hdt_attn_bwd(layout: Layout, q, k, v, o, lse, d_o, softmax_scale: float, dq=None, dk=None, dv=None,
                 workspace=None, stream=None):
    """Returns (dq, dk, dv); dq like q, dk and dv like k."""
    import torch
    B, H, N, D = q.shape
    _check_tensors((q, o, d_o), q.shape)
    _check_tensors((k, v), (B, H, layout.n_kv, D))
    if (B, N) != (layout.batch, layout.n_pos) or any(t.dtype != q.dtype for t in (k, v, o, d_o)):
        raise ValueError("tensor shapes or dtypes do not match the layout")
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(k) if dv is None else dv
    need = hdt_attn_bwd_workspace_bytes(layout, H, D, _dtype_code(q))
    if workspace is None:
        workspace = _scratch(need, q.device, stream)
    _check(load_library().hdt_attn_bwd(layout.handle, _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o),
                                       _ptr(dq), _ptr(dk), _ptr(dv), H, D, _dtype_code(q), float(softmax_scale),
                                       _ptr(workspace), workspace.numel() * workspace.element_size(),
                                       _stream_ptr(stream)))
    return dq, dk, dv


def hdt_attn_bwd_no_alloc(layout: Layout, q, k, v, o, lse, d_o, softmax_scale: float, dq, dk, dv, stream=None):
    """hdt_attn_bwd on the library's own workspace: every tensor, outputs included, comes from the caller, and
    neither this wrapper nor the library allocates device memory.  Returns (dq, dk, dv)."""
    B, H, N, D = q.shape
    _check_tensors((q, o, d_o, dq), q.shape)
    _check_tensors((k, v, dk, dv), (B, H, layout.n_kv, D))
    if (B, N) != (layout.batch, layout.n_pos) or any(t.dtype != q.dtype for t in (k, v, o, d_o, dq, dk, dv)):
        raise ValueError("tensor shapes or dtypes do not match the layout")
    _check(load_library().hdt_attn_bwd_no_alloc(layout.handle, _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o),
                                                _ptr(dq), _ptr(dk), _ptr(dv), H, D, _dtype_code(q),
                                                float(softmax_scale), _stream_ptr(stream)))
    return dq, dk, dv


def hdt_release_cached_memory():
    _check(load_library().hdt_release_cached_memory())


def hdt_timing_enable(enable: bool):
    _check(load_library().hdt_timing_enable(int(enable)))


def hdt_timing_reset():
    _check(load_library().hdt_timing_reset())


def hdt_timing_read() -> dict:
    """{kernel name: (launches, total milliseconds)} since the last reset."""
    cap = 64
    names = (ctypes.c_char_p * cap)()
    launches = (ctypes.c_int64 * cap)()
    ms = (ctypes.c_double * cap)()
    n = load_library().hdt_timing_read(names, launches, ms, cap)
    return {names[i].decode(): (int(launches[i]), float(ms[i])) for i in range(min(n, cap))}


def hdt_probe_mfma_bf16(workgroups: int, iters: int, sink, stream=None) -> float:
    """Enqueues the MFMA measuring kernel (see hdt.h); returns the floating-point operations of the launch."""
    flop = ctypes.c_double(0.0)
    _check(load_library().hdt_probe_mfma_bf16(int(workgroups), int(iters), _ptr(sink), ctypes.byref(flop),
                                              _stream_ptr(stream)))
    return float(flop.value)


def hdt_parents_from_levels(level, out=None, stream=None):
    """level: int32 device tensor [batch][n_pos] of documents laid out with their anchors in front -> parent ids."""
    import torch
    if level.dtype != torch.int32 or level.dim() != 2 or not (level.is_cuda and level.is_contiguous()):
        raise TypeError("level must be a contiguous int32 device tensor [batch][n_pos]")
    B, N = level.shape
    if out is None:
        out = torch.empty_like(level)
    _check(load_library().hdt_parents_from_levels(_ptr(level) if B * N else None, B, N, _ptr(out) if B * N else None,
                                                  _stream_ptr(stream)))
    return out


def hdt_index_vectors(level, parent, n_levels: int, out=None, workspace=None, stream=None):
    """level, parent: int32 device tensors [batch][n_pos] -> int32 device tensor [batch][n_pos][n_levels]."""
    import torch
    if level.dtype != torch.int32 or parent.dtype != torch.int32 or level.shape != parent.shape or level.dim() != 2:
        raise TypeError("level and parent must be int32 [batch][n_pos]")
    if not (level.is_cuda and parent.is_cuda and level.is_contiguous() and parent.is_contiguous()):
        raise ValueError("level and parent must be contiguous device tensors")
    B, N = level.shape
    if out is None:
        out = torch.empty((B, N, n_levels), dtype=torch.int32, device=level.device)
    need = int(load_library().hdt_index_vectors_workspace_bytes(B, N))
    if workspace is None:
        workspace = _scratch(need, level.device, stream)
    _check(load_library().hdt_index_vectors(_ptr(level) if B * N else None, _ptr(parent) if B * N else None, B, N,
                                            n_levels, _ptr(out), _ptr(workspace),
                                            workspace.numel() * workspace.element_size(), _stream_ptr(stream)))
    return out


def hdt_hpe_table(rows: int, d_model: int, device="cuda", stream=None):
    """float32 device tensor [rows][d_model]: the sinusoidal table."""
    import torch
    table = torch.empty((rows, d_model), dtype=torch.float32, device=device)
    _check(load_library().hdt_hpe_table(_ptr(table) if rows else None, rows, d_model, _stream_ptr(stream)))
    return table


def hdt_hpe_add(p, table, x, stream=None):
    """x [batch][n_pos][d_model] (bf16 or fp32 device tensor) += HPE(p), in place.  Returns x."""
    _check_tensors((x,))
    B, N, L = p.shape
    if tuple(x.shape[:2]) != (B, N):
        raise ValueError("x and p disagree on [batch][n_pos]")
    rows = 0 if table is None else table.shape[0]
    _check(load_library().hdt_hpe_add(_ptr(p), B, N, L, _ptr(table) if rows else None, rows, _ptr(x), x.shape[2],
                                      _dtype_code(x), _stream_ptr(stream)))
    return x
