"""Thin Python binding over libloki.so's C ABI (include/loki.h).

Argument marshalling only: torch supplies device memory and the stream, every
step of the path runs in the HIP kernels.  There is no CPU fallback: if the
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libloki.so")

LOKI_F32, LOKI_BF16 = 0, 1
SELECT_PER_QUERY_HEAD, SELECT_PER_KV_GROUP = 0, 1
PATH_SPLIT, PATH_FUSED, PATH_CLUSTER, PATH_MASK = 0x100, 0x200, 0x300, 0x300
WORKSPACE_ZEROED = 0x400
PROFILE_MAX_KERNELS = 8


class LokiError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class Layout(ctypes.Structure):
    """Mirror of ``loki_layout``."""

    _fields_ = [("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("D", ctypes.c_int32), ("d_split", ctypes.c_int32), ("S_cap", ctypes.c_int32),
                ("dtype", ctypes.c_int32)]


_lib = None


def lib() -> ctypes.CDLL:
    """Loads libloki.so (built by ``paper_2406_02542_amd.build``); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2406_02542_amd.build` "
            "(there is no fallback path)")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    LP = ctypes.POINTER(Layout)
    L.loki_version.restype = i32
    L.loki_version.argtypes = []
    L.loki_status_string.restype = ctypes.c_char_p
    L.loki_status_string.argtypes = [i32]
    L.loki_cache_bytes.restype = i32
    L.loki_cache_bytes.argtypes = [LP, ctypes.POINTER(sz), ctypes.POINTER(sz), ctypes.POINTER(sz)]
    L.loki_workspace_bytes.restype = i32
    L.loki_workspace_bytes.argtypes = [LP, i32, i32, i32, i32, ctypes.POINTER(sz)]
    L.loki_rotate_keys.restype = i32
    L.loki_rotate_keys.argtypes = [LP, vp, vp, vp, vp, i32, i32, vp]
    L.loki_rotate_keys_paged.restype = i32
    L.loki_rotate_keys_paged.argtypes = [LP, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp]
    L.loki_decode_attn.restype = i32
    L.loki_decode_attn.argtypes = [LP, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, sz, vp, vp, vp]
    L.loki_decode_attn_static.restype = i32
    L.loki_decode_attn_static.argtypes = [LP, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp]
    L.loki_decode_step.restype = i32
    L.loki_decode_step.argtypes = [LP, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, sz, vp, vp, vp]
    L.dense_decode_step.restype = i32
    L.dense_decode_step.argtypes = [LP, vp, vp, vp, i32, vp, vp, sz, vp, vp]
    L.loki_pca_attn.restype = i32
    L.loki_pca_attn.argtypes = [LP, vp, vp, vp, vp, i32, i32, vp, sz, vp, vp]
    L.loki_pca_workspace_bytes.restype = i32
    L.loki_pca_workspace_bytes.argtypes = [LP, ctypes.c_longlong, ctypes.POINTER(sz)]
    L.loki_pca_fit.restype = i32
    L.loki_pca_fit.argtypes = [LP, vp, ctypes.c_longlong, vp, vp, vp, sz, vp]
    L.loki_rank_at.restype = i32
    L.loki_rank_at.argtypes = [vp, i32, i32, ctypes.c_float, vp, vp]
    L.loki_layer_width.restype = i32
    L.loki_layer_width.argtypes = [vp, i32, i32, ctypes.c_float, i32, vp, vp, vp]
    L.loki_index_jaccard.restype = i32
    L.loki_index_jaccard.argtypes = [vp, vp, i32, i32, vp, vp]
    L.dense_decode_attn.restype = i32
    L.dense_decode_attn.argtypes = [LP, vp, vp, vp, i32, vp, sz, vp, vp]
    L.loki_profile_create.restype = i32
    L.loki_profile_create.argtypes = [ctypes.POINTER(vp)]
    L.loki_profile_destroy.restype = i32
    L.loki_profile_destroy.argtypes = [vp]
    L.loki_profile_attach.restype = i32
    L.loki_profile_attach.argtypes = [vp]
    L.loki_debug_cluster_spin_limit.restype = i32
    L.loki_debug_cluster_spin_limit.argtypes = [ctypes.c_uint]
    L.loki_cluster_gave_up.restype = i32
    L.loki_cluster_gave_up.argtypes = [vp, ctypes.POINTER(i32), vp]
    L.loki_stream_read.restype = i32
    L.loki_stream_read.argtypes = [vp, sz, vp]
    L.loki_profile_read.restype = i32
    L.loki_profile_read.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_float),
                                    ctypes.POINTER(ctypes.c_char_p)]
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().loki_status_string(int(status)).decode()


def version() -> int:
    return lib().loki_version()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise LokiError(status, where)


def make_layout(B: int, Hq: int, Hkv: int, D: int, d_split: int, S_cap: int,
                dtype: torch.dtype) -> Layout:
    if dtype == torch.float32:
        code = LOKI_F32
    elif dtype == torch.bfloat16:
        code = LOKI_BF16
    else:
        raise ValueError(f"unsupported storage dtype {dtype}")
    return Layout(B, Hq, Hkv, D, d_split, S_cap, code)


def _torch_dtype(layout: Layout) -> torch.dtype:
    return torch.float32 if layout.dtype == LOKI_F32 else torch.bfloat16


def _ptr(t: Optional[torch.Tensor], name: str, dtype: Optional[torch.dtype] = None,
         numel: Optional[int] = None) -> Optional[int]:
    """Device pointer of a tensor after checking it is what the C side assumes."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if numel is not None and t.numel() < numel:
        raise ValueError(f"{name} holds {t.numel()} elements, the call reads/writes {numel}")
    return t.data_ptr()


def _stream_ptr(stream) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def loki_cache_bytes(layout: Layout):
    a, b, c = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().loki_cache_bytes(ctypes.byref(layout), ctypes.byref(a), ctypes.byref(b),
                                  ctypes.byref(c)), "loki_cache_bytes")
    return a.value, b.value, c.value


def loki_workspace_bytes(layout: Layout, S: int, d: int, k: int, select_mode: int) -> int:
    n = ctypes.c_size_t()
    _check(lib().loki_workspace_bytes(ctypes.byref(layout), S, d, k, select_mode, ctypes.byref(n)),
           "loki_workspace_bytes")
    return n.value


def alloc_cache(layout: Layout, device="cuda"):
    """Allocates (klo, khi, v) tensors of the layout's shape (zero-filled)."""
    dt = _torch_dtype(layout)
    B, H, S, D, d = layout.B, layout.Hkv, layout.S_cap, layout.D, layout.d_split
    klo = torch.zeros((B, H, S, d), dtype=dt, device=device)
    khi = torch.zeros((B, H, S, D - d), dtype=dt, device=device) if d < D else None
    v = torch.zeros((B, H, S, D), dtype=dt, device=device)
    return klo, khi, v


def alloc_workspace(layout: Layout, S: int, d: int, k: int, select_mode: int,
                    device="cuda", zeroed: bool = False) -> torch.Tensor:
    """zeroed: a workspace filled with zeros, which the caller may then pass with WORKSPACE_ZEROED."""
    n = loki_workspace_bytes(layout, S, d, k, select_mode)
    make = torch.zeros if zeroed else torch.empty
    return make(max(n, 256), dtype=torch.uint8, device=device)


def loki_rotate_keys(layout: Layout, k_new: torch.Tensor, P: torch.Tensor, klo: torch.Tensor,
                     khi: Optional[torch.Tensor], pos: int, n_new: int, stream=None) -> None:
    dt = _torch_dtype(layout)
    rows = layout.B * layout.Hkv
    _check(lib().loki_rotate_keys(
        ctypes.byref(layout),
        _ptr(k_new, "k_new", dt, rows * n_new * layout.D),
        _ptr(P, "P", torch.float32, layout.Hkv * layout.D * layout.D),
        _ptr(klo, "klo", dt, rows * layout.S_cap * layout.d_split),
        _ptr(khi, "khi", dt, rows * layout.S_cap * (layout.D - layout.d_split)),
        pos, n_new, _stream_ptr(stream)), "loki_rotate_keys")


def loki_rotate_keys_paged(layout: Layout, k_new: torch.Tensor, P: torch.Tensor, klo: torch.Tensor,
                           khi: Optional[torch.Tensor], page_table: torch.Tensor, page_rows: int,
                           n_pages: int, pos: int, n_new: int, stream=None) -> None:
    dt = _torch_dtype(layout)
    rows = layout.B * layout.Hkv
    pool_rows = n_pages * layout.Hkv * page_rows
    _check(lib().loki_rotate_keys_paged(
        ctypes.byref(layout),
        _ptr(k_new, "k_new", dt, rows * n_new * layout.D),
        _ptr(P, "P", torch.float32, layout.Hkv * layout.D * layout.D),
        _ptr(klo, "klo", dt, pool_rows * layout.d_split),
        _ptr(khi, "khi", dt, pool_rows * (layout.D - layout.d_split)),
        _ptr(page_table, "page_table", torch.int32, layout.B),
        page_rows, page_table.numel() // layout.B, n_pages, pos, n_new,
        _stream_ptr(stream)), "loki_rotate_keys_paged")


def loki_decode_attn(layout: Layout, q: torch.Tensor, P: torch.Tensor, klo: torch.Tensor,
                     khi: Optional[torch.Tensor], v: torch.Tensor, S: int, d: int, k: int,
                     select_mode: int, workspace: torch.Tensor, out: torch.Tensor,
                     out_idx: Optional[torch.Tensor] = None, stream=None) -> None:
    dt = _torch_dtype(layout)
    rows = layout.B * layout.Hkv
    nq = layout.B * layout.Hq * layout.D
    hsel = layout.Hq if (select_mode & ~(PATH_MASK | WORKSPACE_ZEROED)) == SELECT_PER_QUERY_HEAD else layout.Hkv
    _check(lib().loki_decode_attn(
        ctypes.byref(layout),
        _ptr(q, "q", dt, nq),
        _ptr(P, "P", torch.float32, layout.Hkv * layout.D * layout.D),
        _ptr(klo, "klo", dt, rows * layout.S_cap * layout.d_split),
        _ptr(khi, "khi", dt, rows * layout.S_cap * (layout.D - layout.d_split)),
        _ptr(v, "v", dt, rows * layout.S_cap * layout.D),
        S, d, k, select_mode,
        _ptr(workspace, "workspace", torch.uint8), workspace.numel(),
        _ptr(out, "out", dt, nq),
        _ptr(out_idx, "out_idx", torch.int32, layout.B * hsel * k),
        _stream_ptr(stream)), "loki_decode_attn")


STATIC_SCRATCH_BYTES = 64 << 20


def loki_decode_attn_static(layout: Layout, q: torch.Tensor, P: torch.Tensor, klo: torch.Tensor,
                            khi: Optional[torch.Tensor], v: torch.Tensor, S: int, d: int, k: int,
                            select_mode: int, out: torch.Tensor,
                            out_idx: Optional[torch.Tensor] = None, stream=None) -> None:
    """loki_decode_attn on the library's built-in scratch buffer (no workspace argument)."""
    dt = _torch_dtype(layout)
    rows = layout.B * layout.Hkv
    nq = layout.B * layout.Hq * layout.D
    hsel = layout.Hq if (select_mode & ~(PATH_MASK | WORKSPACE_ZEROED)) == SELECT_PER_QUERY_HEAD else layout.Hkv
    _check(lib().loki_decode_attn_static(
        ctypes.byref(layout),
        _ptr(q, "q", dt, nq),
        _ptr(P, "P", torch.float32, layout.Hkv * layout.D * layout.D),
        _ptr(klo, "klo", dt, rows * layout.S_cap * layout.d_split),
        _ptr(khi, "khi", dt, rows * layout.S_cap * (layout.D - layout.d_split)),
        _ptr(v, "v", dt, rows * layout.S_cap * layout.D),
        S, d, k, select_mode,
        _ptr(out, "out", dt, nq),
        _ptr(out_idx, "out_idx", torch.int32, layout.B * hsel * k),
        _stream_ptr(stream)), "loki_decode_attn_static")


class StepArgs(ctypes.Structure):
    """Mirror of ``loki_step_args``."""
    _fields_ = [("seq_lens", ctypes.c_void_p), ("ks", ctypes.c_void_p),
                ("k_new", ctypes.c_void_p), ("v_new", ctypes.c_void_p),
                ("queries_per_seq", ctypes.c_int32), ("page_rows", ctypes.c_int32),
                ("page_table", ctypes.c_void_p), ("pages_per_seq", ctypes.c_int32),
                ("n_pages", ctypes.c_int32)]


def loki_decode_step(layout: Layout, q: torch.Tensor, P: torch.Tensor, klo: torch.Tensor,
                     khi: Optional[torch.Tensor], v: torch.Tensor, S_max: int, d: int, k_max: int,
                     select_mode: int, workspace: torch.Tensor, out: torch.Tensor,
                     out_idx: Optional[torch.Tensor] = None, seq_lens: Optional[torch.Tensor] = None,
                     ks: Optional[torch.Tensor] = None, k_new: Optional[torch.Tensor] = None,
                     v_new: Optional[torch.Tensor] = None, queries_per_seq: int = 1,
                     page_table: Optional[torch.Tensor] = None, page_rows: int = 0,
                     n_pages: int = 0, stream=None) -> None:
    """With ``page_table`` [B, pages_per_seq] (int32), ``klo``/``khi``/``v`` are the paged
    pools [n_pages, Hkv, page_rows, width]."""
    dt = _torch_dtype(layout)
    m = max(1, queries_per_seq)
    rows = layout.B * layout.Hkv
    nq = layout.B * m * layout.Hq * layout.D
    hsel = layout.Hq if (select_mode & ~(PATH_MASK | WORKSPACE_ZEROED)) == SELECT_PER_QUERY_HEAD else layout.Hkv
    args = StepArgs(
        _ptr(seq_lens, "seq_lens", torch.int32, layout.B * m),
        _ptr(ks, "ks", torch.int32, layout.B * m),
        _ptr(k_new, "k_new", dt, rows * m * layout.D),
        _ptr(v_new, "v_new", dt, rows * m * layout.D),
        queries_per_seq, page_rows,
        _ptr(page_table, "page_table", torch.int32, layout.B),
        (page_table.numel() // layout.B) if page_table is not None else 0, n_pages)
    cache_rows = (n_pages * layout.Hkv * page_rows) if page_table is not None else rows * layout.S_cap
    _check(lib().loki_decode_step(
        ctypes.byref(layout),
        _ptr(q, "q", dt, nq),
        _ptr(P, "P", torch.float32, layout.Hkv * layout.D * layout.D),
        _ptr(klo, "klo", dt, cache_rows * layout.d_split),
        _ptr(khi, "khi", dt, cache_rows * (layout.D - layout.d_split)),
        _ptr(v, "v", dt, cache_rows * layout.D),
        S_max, d, k_max, select_mode, ctypes.byref(args),
        _ptr(workspace, "workspace", torch.uint8), workspace.numel(),
        _ptr(out, "out", dt, nq),
        _ptr(out_idx, "out_idx", torch.int32, layout.B * m * hsel * k_max),
        _stream_ptr(stream)), "loki_decode_step")


def dense_decode_step(layout: Layout, q: torch.Tensor, k_full: torch.Tensor, v: torch.Tensor,
                      S_max: int, seq_lens: Optional[torch.Tensor],
                      workspace: Optional[torch.Tensor], out: torch.Tensor, stream=None) -> None:
    dt = _torch_dtype(layout)
    rows = layout.B * layout.Hkv
    nq = layout.B * layout.Hq * layout.D
    _check(lib().dense_decode_step(
        ctypes.byref(layout),
        _ptr(q, "q", dt, nq),
        _ptr(k_full, "k_full", dt, rows * layout.S_cap * layout.D),
        _ptr(v, "v", dt, rows * layout.S_cap * layout.D),
        S_max,
        _ptr(seq_lens, "seq_lens", torch.int32, layout.B),
        _ptr(workspace, "workspace", torch.uint8),
        workspace.numel() if workspace is not None else 0,
        _ptr(out, "out", dt, nq),
        _stream_ptr(stream)), "dense_decode_step")


def dense_decode_attn(layout: Layout, q: torch.Tensor, k_full: torch.Tensor, v: torch.Tensor,
                      S: int, workspace: Optional[torch.Tensor], out: torch.Tensor,
                      stream=None) -> None:
    dt = _torch_dtype(layout)
    rows = layout.B * layout.Hkv
    nq = layout.B * layout.Hq * layout.D
    _check(lib().dense_decode_attn(
        ctypes.byref(layout),
        _ptr(q, "q", dt, nq),
        _ptr(k_full, "k_full", dt, rows * layout.S_cap * layout.D),
        _ptr(v, "v", dt, rows * layout.S_cap * layout.D),
        S,
        _ptr(workspace, "workspace", torch.uint8),
        workspace.numel() if workspace is not None else 0,
        _ptr(out, "out", dt, nq),
        _stream_ptr(stream)), "dense_decode_attn")


def loki_pca_attn(layout: Layout, q: torch.Tensor, P: torch.Tensor, klo: torch.Tensor,
                  v: torch.Tensor, S: int, d: int, workspace: torch.Tensor, out: torch.Tensor,
                  stream=None) -> None:
    dt = _torch_dtype(layout)
    rows = layout.B * layout.Hkv
    nq = layout.B * layout.Hq * layout.D
    _check(lib().loki_pca_attn(
        ctypes.byref(layout),
        _ptr(q, "q", dt, nq),
        _ptr(P, "P", torch.float32, layout.Hkv * layout.D * layout.D),
        _ptr(klo, "klo", dt, rows * layout.S_cap * layout.d_split),
        _ptr(v, "v", dt, rows * layout.S_cap * layout.D),
        S, d,
        _ptr(workspace, "workspace", torch.uint8), workspace.numel(),
        _ptr(out, "out", dt, nq),
        _stream_ptr(stream)), "loki_pca_attn")


def loki_pca_workspace_bytes(layout: Layout, n_rows: int) -> int:
    n = ctypes.c_size_t()
    _check(lib().loki_pca_workspace_bytes(ctypes.byref(layout), n_rows, ctypes.byref(n)),
           "loki_pca_workspace_bytes")
    return n.value


def loki_pca_fit(layout: Layout, keys: torch.Tensor, n_rows: int, P: torch.Tensor,
                 eigenvalues: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    dt = _torch_dtype(layout)
    _check(lib().loki_pca_fit(
        ctypes.byref(layout),
        _ptr(keys, "keys", dt, layout.Hkv * n_rows * layout.D), n_rows,
        _ptr(P, "P", torch.float32, layout.Hkv * layout.D * layout.D),
        _ptr(eigenvalues, "eigenvalues", torch.float32, layout.Hkv * layout.D),
        _ptr(workspace, "workspace", torch.uint8), workspace.numel(),
        _stream_ptr(stream)), "loki_pca_fit")


def loki_rank_at(eigenvalues: torch.Tensor, v_percent: float, ranks: torch.Tensor, stream=None) -> None:
    n, D = eigenvalues.shape
    _check(lib().loki_rank_at(_ptr(eigenvalues, "eigenvalues", torch.float32, n * D), n, D, v_percent,
                              _ptr(ranks, "ranks", torch.int32, n), _stream_ptr(stream)), "loki_rank_at")


def loki_layer_width(eigenvalues: torch.Tensor, v_percent: float, multiple: int,
                     mean_rank: Optional[torch.Tensor], d_out: torch.Tensor, stream=None) -> None:
    n, D = eigenvalues.shape
    _check(lib().loki_layer_width(_ptr(eigenvalues, "eigenvalues", torch.float32, n * D), n, D, v_percent,
                                  multiple, _ptr(mean_rank, "mean_rank", torch.float32, 1),
                                  _ptr(d_out, "d_out", torch.int32, 1), _stream_ptr(stream)),
           "loki_layer_width")


def loki_index_jaccard(idx_a: torch.Tensor, idx_b: torch.Tensor, out: torch.Tensor, stream=None) -> None:
    k = idx_a.shape[-1]
    n = idx_a.numel() // k
    _check(lib().loki_index_jaccard(_ptr(idx_a, "idx_a", torch.int32, n * k),
                                    _ptr(idx_b, "idx_b", torch.int32, n * k), n, k,
                                    _ptr(out, "out", torch.float32, n), _stream_ptr(stream)),
           "loki_index_jaccard")


def loki_debug_cluster_spin_limit(polls: int) -> None:
    """Sets how many polls a block of a PATH_CLUSTER launch waits for its unit's other blocks
    (0 restores the default)."""
    _check(lib().loki_debug_cluster_spin_limit(int(polls)), "loki_debug_cluster_spin_limit")


def loki_cluster_gave_up(workspace: torch.Tensor, stream=None) -> bool:
    """True if a PATH_CLUSTER launch on this workspace gave up waiting since its control words
    were last cleared (synchronises with the stream)."""
    flag = ctypes.c_int32(0)
    _check(lib().loki_cluster_gave_up(ctypes.c_void_p(workspace.data_ptr()), ctypes.byref(flag),
                                      _stream_ptr(stream)), "loki_cluster_gave_up")
    return bool(flag.value)


def loki_stream_read(buf: torch.Tensor, nbytes: int, stream=None) -> None:
    """Enqueues the library's trivial read kernel over the first ``nbytes`` bytes of ``buf``."""
    if not buf.is_cuda or not buf.is_contiguous() or nbytes > buf.numel() * buf.element_size():
        raise ValueError("buf must be a contiguous device tensor of at least nbytes bytes")
    _check(lib().loki_stream_read(ctypes.c_void_p(buf.data_ptr()), nbytes, _stream_ptr(stream)),
           "loki_stream_read")


class Profile:
    """Owns a ``loki_profile``; while attached, every library call made from this
    thread records HIP events around each kernel it launches."""

    def __init__(self):
        h = ctypes.c_void_p()
        _check(lib().loki_profile_create(ctypes.byref(h)), "loki_profile_create")
        self._h = h

    def attach(self):
        _check(lib().loki_profile_attach(self._h), "loki_profile_attach")

    @staticmethod
    def detach():
        _check(lib().loki_profile_attach(None), "loki_profile_attach")

    def read(self):
        """[(kernel name, milliseconds)] of the most recent profiled call."""
        n = ctypes.c_int()
        ms = (ctypes.c_float * PROFILE_MAX_KERNELS)()
        names = (ctypes.c_char_p * PROFILE_MAX_KERNELS)()
        _check(lib().loki_profile_read(self._h, ctypes.byref(n), ms, names), "loki_profile_read")
        return [(names[i].decode(), float(ms[i])) for i in range(n.value)]

    def close(self):
        if self._h is not None:
            lib().loki_profile_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
