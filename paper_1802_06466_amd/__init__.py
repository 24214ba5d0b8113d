"""Thin Python binding of the RBE retrieval library (include/rbe.h, include/rbe_debug.h).

Argument marshalling only: every step of the path runs in the HIP kernels of
``librbe_hip.so``.  There is no CPU fallback -- importing works without the
library (so that CPU-only tooling can inspect the package), but any call raises
``RuntimeError`` if the shared library has not been built.

Function names match the C ABI.  Host arrays are numpy arrays; device arrays
are torch tensors (used for device memory and streams only).
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

from . import _build

RBE_OK, RBE_EINVAL, RBE_ENOMEM, RBE_EHIP, RBE_ESTATE, RBE_EUNSUPPORTED = 0, -1, -2, -3, -4, -5
RBE_MEM_HOST, RBE_MEM_DEVICE = 0, 1
RBE_BORROW = 1 << 0
RBE_COSINE = 1 << 1
RBE_DYADIC = 1 << 2
RBE_SELECT_EXACT, RBE_SELECT_NEARLOSSLESS, RBE_SELECT_NEARLOSSLESS_Q2 = 0, 1, 2
RBE_MAX_PLANES, RBE_MAX_QUERIES, RBE_MAX_K, RBE_MAX_LEVELS = 4, 64, 4096, 8
RBE_MAX_ITEMS = 4294966272
RBE_STATIC_SCRATCH_BYTES = 16777216

LIB_PATH = os.environ.get("RBE_HIP_LIB", _build.LIB)   # override: experiments with alternative builds


class RbeError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"rbe error {code}: {message}")
        self.code = code


class rbe_search_stats(ctypes.Structure):
    _fields_ = [
        ("n_levels", ctypes.c_uint32),
        ("fallback", ctypes.c_uint32),
        ("grid_blocks", ctypes.c_uint32),
        ("deep_rows", ctypes.c_uint32),
        ("items_scanned", ctypes.c_uint64 * RBE_MAX_LEVELS),
        ("candidates_max", ctypes.c_uint64 * RBE_MAX_LEVELS),
        ("scan_ms", ctypes.c_float * RBE_MAX_LEVELS),
        ("select_ms", ctypes.c_float * RBE_MAX_LEVELS),
        ("total_gpu_ms", ctypes.c_float),
        ("deep_units", ctypes.c_uint32),
        ("scan_kernel", ctypes.c_uint32 * RBE_MAX_LEVELS),
        ("last_level_parts", ctypes.c_uint32),
        ("deep_rows_level", ctypes.c_uint32 * RBE_MAX_LEVELS),
        ("reserved", ctypes.c_uint32),
    ]


KERNEL_NAMES = {0: "none", 1: "scan_exact", 2: "scan_exact_prog", 3: "scan_exact_prog_hint", 4: "scan_batch_mfma",
                5: "scan_groupmax", 6: "scan_exact_fq", 7: "scan_exact_fq_prog", 8: "scan_exact_prog2_hint", 9: "scan_exact_fq_prog2_hint"}


_lib = None

_u64, _u32, _i32, _vp = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int, ctypes.c_void_p

# name -> (restype, argtypes); the single source for ctypes prototypes
PROTOTYPES = {
    "rbe_index_create": (_i32, [ctypes.POINTER(_vp), _u64, _u32, _u32, _u32]),
    "rbe_index_create_ex": (_i32, [ctypes.POINTER(_vp), _u64, _u32, _u32, _u32, _u32]),
    "rbe_index_bytes": (ctypes.c_size_t, [_u64, _u32, _u32, _u32, _u32]),
    "rbe_index_create_in": (_i32, [ctypes.POINTER(_vp), _u64, _u32, _u32, _u32, _u32, _vp, ctypes.c_size_t]),
    "rbe_load_chunk": (_i32, [_vp, _u64, _u64, _vp, _vp, _i32, _vp]),
    "rbe_encode_chunk": (_i32, [_vp, _u64, _u64, _vp, _i32, _vp]),
    "rbe_encode_corpus": (_i32, [ctypes.POINTER(_vp), _vp, _u64, _u32, _u32, _i32, _u32, _vp]),
    "rbe_finalize": (_i32, [_vp, _vp]),
    "rbe_load_corpus": (_i32, [ctypes.POINTER(_vp), _vp, _vp, _u64, _u32, _u32, _i32, _u32, _vp]),
    "rbe_free": (None, [_vp]),
    "rbe_encode_query": (_i32, [_vp, _u32, _u32, _vp, _vp]),
    "rbe_search": (_i32, [_vp, _vp, _vp, _u32, _u32, _u32, _u32, _u32, _vp, _vp, _vp]),
    "rbe_search_static": (_i32, [_vp, _vp, _vp, _u32, _u32, _u32, _u32, _u32, _vp, _vp, _vp]),
    "rbe_workspace_bytes": (ctypes.c_size_t, [_vp, _u32, _u32, _u32]),
    "rbe_set_workspace": (_i32, [_vp, _vp, ctypes.c_size_t]),
    "rbe_debug_index_info": (_i32, [_vp, _vp]),
    "rbe_debug_issue_rate": (_i32, [_vp, _vp, _vp, _u32, _u32, _u32, _u32, _vp, _vp, _vp]),
    "rbe_search_float": (_i32, [_vp, _vp, _u32, _u32, _u32, _u32, _vp, _vp, _vp]),
    "rbe_debug_scores_float": (_i32, [_vp, _vp, _u64, _u64, _vp, _vp]),
    "rbe_set_profiling": (_i32, [_vp, _i32]),
    "rbe_get_search_stats": (_i32, [_vp, ctypes.POINTER(rbe_search_stats)]),
    "rbe_set_tuning": (_i32, [_vp, _u32, _u32]),
    "rbe_debug_tile_to_phys": (_u32, [_u32, _u32, _u32]),
    "rbe_debug_phys_to_tile": (_u32, [_u32, _u32, _u32]),
    "rbe_debug_set_batch_path": (_i32, [_vp, _i32]),
    "rbe_debug_set_nearlossless_path": (_i32, [_vp, _i32]),
    "rbe_debug_set_progressive": (_i32, [_vp, _i32]),
    "rbe_debug_set_plan_split": (_i32, [_vp, _i32]),
    "rbe_debug_query_mass": (_i32, [_vp, _vp, _u32, _u32, _u32, _vp]),
    "rbe_debug_exact_plan": (_i32, [_u64, _u32, _u32, _u32, _vp, _vp, _vp]),
    "rbe_debug_batch_operands": (_i32, [_vp, _vp, _vp, _u32, _u32, _u32, _u32, _u32, _vp, ctypes.c_size_t, _vp, _vp, _vp]),
    "rbe_debug_batch_operands_i8": (_i32, [_vp, _vp, _vp, _u32, _u32, _u32, _vp, ctypes.c_size_t, _vp, _vp, _vp, _vp]),
    "rbe_debug_batch_operands_i8_dyadic": (_i32, [_vp, _u32, _u32, _u32, _u32, _vp, ctypes.c_size_t, _vp, _vp, _vp]),
    "rbe_debug_popcounts": (_i32, [_vp, _vp, _u32, _u64, _u64, _vp, _vp]),
    "rbe_debug_scores": (_i32, [_vp, _vp, _vp, _u32, _u64, _u64, _vp, _vp]),
    "rbe_debug_read_scales": (_i32, [_vp, _u64, _u64, _vp, _vp]),
    "rbe_debug_read_planes": (_i32, [_vp, _u64, _u64, _vp, _vp]),
    "rbe_debug_copy": (_i32, [_vp, _vp, ctypes.c_size_t, _vp]),
    "rbe_debug_read": (_i32, [_vp, ctypes.c_size_t, _vp, ctypes.c_size_t, _vp]),
    "rbe_strerror": (ctypes.c_char_p, [_i32]),
    "rbe_last_error": (ctypes.c_char_p, []),
    "rbe_n_items": (_u64, [_vp]),
    "rbe_dim": (_u32, [_vp]),
    "rbe_n_planes": (_u32, [_vp]),
}


def load_library():
    """dlopen librbe_hip.so (built in-tree by ``_build.build``).  Raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it first (python -m paper_1802_06466_amd._build "
                "or __graft_entry__.build()); there is no CPU fallback")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in PROTOTYPES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _check(code: int):
    if code != RBE_OK:
        lib = load_library()
        raise RbeError(code, f"{lib.rbe_strerror(code).decode()}: {lib.rbe_last_error().decode()}")


def _stream_ptr(stream) -> Optional[int]:
    """hipStream_t of a torch stream; None -> torch's current stream if torch has a
    GPU context, else the default stream."""
    if stream is not None:
        return int(stream.cuda_stream) if hasattr(stream, "cuda_stream") else int(stream)
    try:
        import torch
        if torch.cuda.is_available():
            return int(torch.cuda.current_stream().cuda_stream)
    except ImportError:
        pass
    return None


def _host(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data_as(_vp)


class Index:
    """Owner of an ``rbe_index*``."""

    def __init__(self, handle: int, keep=None):
        self._h = _vp(handle)
        self._keep = keep           # tensors whose memory the index uses (caller-owned storage / workspace)
        self._ws = None

    @property
    def handle(self):
        if not self._h:
            raise RbeError(RBE_ESTATE, "index already freed")
        return self._h

    @property
    def n_items(self) -> int:
        return int(load_library().rbe_n_items(self.handle))

    @property
    def dim(self) -> int:
        return int(load_library().rbe_dim(self.handle))

    @property
    def n_planes(self) -> int:
        return int(load_library().rbe_n_planes(self.handle))

    def free(self):
        if self._h:
            load_library().rbe_free(self._h)
            self._h = _vp(None)

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def _corpus_ptrs(planes, scales, n_planes: int, count: int, W: int):
    """(planes_ptr, scales_ptr, mem_kind, keepalive) for numpy arrays or torch tensors.
    scales may be None (dyadic indexes take no scales)."""
    if isinstance(planes, np.ndarray) or isinstance(scales, np.ndarray):
        p, pp = _host(planes, np.uint64)
        if p.shape != (n_planes, count, W):
            raise RbeError(RBE_EINVAL, f"expected planes {(n_planes, count, W)}, got {p.shape}")
        if scales is None:
            return pp, None, RBE_MEM_HOST, (p,)
        s, sp = _host(scales, np.float32)
        if s.shape != (n_planes, count):
            raise RbeError(RBE_EINVAL, f"expected scales {(n_planes, count)}, got {s.shape}")
        return pp, sp, RBE_MEM_HOST, (p, s)
    import torch
    if not isinstance(planes, torch.Tensor) or not (scales is None or isinstance(scales, torch.Tensor)):
        raise RbeError(RBE_EINVAL, "planes/scales must both be numpy arrays or both torch tensors")
    if planes.dtype not in (torch.int64, torch.uint64) or tuple(planes.shape) != (n_planes, count, W):
        raise RbeError(RBE_EINVAL, "planes must be int64/uint64 of shape [P][count][W]")
    planes = planes.contiguous()
    kind = RBE_MEM_DEVICE if planes.is_cuda else RBE_MEM_HOST
    if scales is None:
        return _vp(planes.data_ptr()), None, kind, (planes,)
    if scales.dtype != torch.float32 or tuple(scales.shape) != (n_planes, count):
        raise RbeError(RBE_EINVAL, "scales must be float32 of shape [P][count]")
    if planes.device != scales.device:
        raise RbeError(RBE_EINVAL, "planes and scales live on different devices")
    scales = scales.contiguous()
    return _vp(planes.data_ptr()), _vp(scales.data_ptr()), kind, (planes, scales)


def rbe_index_create(n_items: int, dim: int, n_planes: int, flags: int = 0) -> Index:
    out = _vp(None)
    _check(load_library().rbe_index_create(ctypes.byref(out), n_items, dim, n_planes, flags))
    return Index(out.value)


def rbe_index_create_ex(n_items: int, dim: int, n_planes: int, flags: int = 0, sample_ratio: int = 0) -> Index:
    out = _vp(None)
    _check(load_library().rbe_index_create_ex(ctypes.byref(out), n_items, dim, n_planes, flags, sample_ratio))
    return Index(out.value)


def rbe_index_bytes(n_items: int, dim: int, n_planes: int, flags: int = 0, sample_ratio: int = 0) -> int:
    return int(load_library().rbe_index_bytes(n_items, dim, n_planes, flags, sample_ratio))


def rbe_index_create_in(n_items: int, dim: int, n_planes: int, flags: int, sample_ratio: int, storage) -> Index:
    """Index inside `storage`, a torch cuda tensor (any dtype) of at least rbe_index_bytes(...) bytes.
    The Index object keeps a reference to the tensor."""
    if not getattr(storage, "is_cuda", False):
        raise RbeError(RBE_EINVAL, "storage must be a torch cuda tensor")
    out = _vp(None)
    _check(load_library().rbe_index_create_in(ctypes.byref(out), n_items, dim, n_planes, flags, sample_ratio,
                                              _vp(storage.data_ptr()), storage.numel() * storage.element_size()))
    return Index(out.value, keep=storage)


def rbe_workspace_bytes(ix: Index, n_queries: int, k: int, mode: int = RBE_SELECT_EXACT) -> int:
    return int(load_library().rbe_workspace_bytes(ix.handle, n_queries, k, mode))


def rbe_set_workspace(ix: Index, workspace):
    """workspace: a torch cuda tensor that will hold all device scratch of later searches, or None to
    return to library-owned scratch.  The Index object keeps a reference to the tensor."""
    if workspace is None:
        _check(load_library().rbe_set_workspace(ix.handle, None, 0))
    else:
        if not getattr(workspace, "is_cuda", False):
            raise RbeError(RBE_EINVAL, "workspace must be a torch cuda tensor")
        _check(load_library().rbe_set_workspace(ix.handle, _vp(workspace.data_ptr()),
                                                workspace.numel() * workspace.element_size()))
    ix._ws = workspace


def rbe_debug_issue_rate(ix: Index, q_planes, q_scales, kernel: int, repeat: int, stream=None):
    """(ms, pairs) of one launch of a batch scan going over its tiles 1 + repeat times without reloading them
    (kernel 0 = XOR/popcount batch scan, 1 = matrix-core scan): the kernel's instruction mix free of memory traffic."""
    qp, qpp = _host(q_planes, np.uint64)
    Q, Pq = qp.shape[:2]
    qsp = None
    if q_scales is not None:
        qs, qsp = _host(q_scales, np.float32)
    ms = ctypes.c_float(0.0)
    pairs = ctypes.c_uint64(0)
    _check(load_library().rbe_debug_issue_rate(ix.handle, qpp, qsp, Q, Pq, kernel, repeat, ctypes.byref(ms),
                                               ctypes.byref(pairs), _stream_ptr(stream)))
    return float(ms.value), int(pairs.value)


def rbe_debug_index_info(ix: Index) -> dict:
    out = np.zeros(4, dtype=np.uint32)
    _check(load_library().rbe_debug_index_info(ix.handle, out.ctypes.data_as(_vp)))
    return {"can_prune": bool(out[0]), "scale_copies": bool(out[1]), "borrowed": bool(out[2]), "caller_workspace": bool(out[3])}


def rbe_load_chunk(ix: Index, first_item: int, planes, scales, stream=None):
    count = int(planes.shape[1])
    pp, sp, kind, keep = _corpus_ptrs(planes, scales, ix.n_planes, count, ix.dim // 64)
    _check(load_library().rbe_load_chunk(ix.handle, first_item, count, pp, sp, kind, _stream_ptr(stream)))
    if kind == RBE_MEM_DEVICE:
        import torch
        torch.cuda.current_stream().synchronize() if stream is None else stream.synchronize()
    del keep


def _vectors_ptr(x, dim: int):
    """(ptr, mem_kind, count, keepalive) for a [count][dim] float32 numpy array or torch tensor."""
    if isinstance(x, np.ndarray):
        a, ap = _host(x, np.float32)
        if a.ndim != 2 or a.shape[1] != dim:
            raise RbeError(RBE_EINVAL, f"expected x [count][{dim}], got {a.shape}")
        return ap, RBE_MEM_HOST, a.shape[0], a
    import torch
    if not isinstance(x, torch.Tensor) or x.dtype != torch.float32 or x.dim() != 2 or x.shape[1] != dim:
        raise RbeError(RBE_EINVAL, f"expected x float32 [count][{dim}]")
    x = x.contiguous()
    return _vp(x.data_ptr()), (RBE_MEM_DEVICE if x.is_cuda else RBE_MEM_HOST), int(x.shape[0]), x


def rbe_encode_chunk(ix: Index, first_item: int, x, stream=None):
    xp, kind, count, keep = _vectors_ptr(x, ix.dim)
    _check(load_library().rbe_encode_chunk(ix.handle, first_item, count, xp, kind, _stream_ptr(stream)))
    if kind == RBE_MEM_DEVICE:
        import torch
        torch.cuda.current_stream().synchronize() if stream is None else stream.synchronize()
    del keep


def rbe_encode_corpus(x, n_planes: int, flags: int = 0, stream=None) -> Index:
    """x [N][dim] float32 (numpy = host, torch cuda = device) -> searchable index."""
    dim = int(x.shape[1])
    xp, kind, count, keep = _vectors_ptr(x, dim)
    out = _vp(None)
    _check(load_library().rbe_encode_corpus(ctypes.byref(out), xp, count, dim, n_planes, kind, flags,
                                            _stream_ptr(stream)))
    del keep
    return Index(out.value)


def rbe_finalize(ix: Index, stream=None):
    _check(load_library().rbe_finalize(ix.handle, _stream_ptr(stream)))


def rbe_load_corpus(planes, scales, flags: int = 0, stream=None) -> Index:
    """planes [P][N][W] uint64, scales [P][N] float32 or None for RBE_DYADIC
    (numpy = host, torch cuda = device)."""
    P, N, W = (int(v) for v in planes.shape)
    pp, sp, kind, keep = _corpus_ptrs(planes, scales, P, N, W)
    out = _vp(None)
    _check(load_library().rbe_load_corpus(ctypes.byref(out), pp, sp, N, 64 * W, P, kind, flags, _stream_ptr(stream)))
    del keep
    return Index(out.value)


def rbe_free(ix: Index):
    ix.free()


def rbe_encode_query(x, n_planes: int):
    """x [dim] float32 -> (planes uint64 [n_planes][dim/64], scales float32 [n_planes])."""
    x, xp = _host(x, np.float32)
    if x.ndim != 1:
        raise RbeError(RBE_EINVAL, "x must be one vector")
    dim = x.shape[0]
    planes = np.zeros((n_planes, max(dim // 64, 1)), dtype=np.uint64)
    scales = np.zeros(n_planes, dtype=np.float32)
    _check(load_library().rbe_encode_query(xp, dim, n_planes, planes.ctypes.data_as(_vp), scales.ctypes.data_as(_vp)))
    return planes, scales


def rbe_search_static(ix: Index, q_planes, q_scales, k: int, mode: int = RBE_SELECT_EXACT, group_size_I: int = 0,
                      stream=None):
    """rbe_search on the library's fixed scratch array (no device allocation in the call)."""
    return rbe_search(ix, q_planes, q_scales, k, mode, group_size_I, stream, _entry="rbe_search_static")


def rbe_search(ix: Index, q_planes, q_scales, k: int, mode: int = RBE_SELECT_EXACT, group_size_I: int = 0,
               stream=None, _entry: str = "rbe_search"):
    """q_planes [Q][Pq][W] uint64, q_scales [Q][Pq] float32 -> (ids int64 [Q][k], scores float32 [Q][k])."""
    qp, qpp = _host(q_planes, np.uint64)
    if qp.ndim != 3 or qp.shape[2] != ix.dim // 64:
        raise RbeError(RBE_EINVAL, f"expected q_planes [Q][Pq][{ix.dim // 64}], got {qp.shape}")
    Q, Pq = qp.shape[:2]
    qsp = None
    if q_scales is not None:
        qs, qsp = _host(q_scales, np.float32)
        if qs.shape != (Q, Pq):
            raise RbeError(RBE_EINVAL, f"expected q_scales {(Q, Pq)}, got {qs.shape}")
    ids = np.empty((Q, max(k, 0)), dtype=np.int64)
    scores = np.empty((Q, max(k, 0)), dtype=np.float32)
    _check(getattr(load_library(), _entry)(ix.handle, qpp, qsp, Q, Pq, k, mode, group_size_I,
                                           ids.ctypes.data_as(_vp), scores.ctypes.data_as(_vp), _stream_ptr(stream)))
    return ids, scores


def rbe_search_float(ix: Index, q, k: int, mode: int = RBE_SELECT_EXACT, group_size_I: int = 0, stream=None):
    """q [Q][dim] float32 -> (ids int64 [Q][k], scores float32 [Q][k]); hybrid scoring."""
    qa, qap = _host(q, np.float32)
    if qa.ndim != 2 or qa.shape[1] != ix.dim:
        raise RbeError(RBE_EINVAL, f"expected q [Q][{ix.dim}], got {qa.shape}")
    Q = qa.shape[0]
    ids = np.empty((Q, max(k, 0)), dtype=np.int64)
    scores = np.empty((Q, max(k, 0)), dtype=np.float32)
    _check(load_library().rbe_search_float(ix.handle, qap, Q, k, mode, group_size_I, ids.ctypes.data_as(_vp),
                                           scores.ctypes.data_as(_vp), _stream_ptr(stream)))
    return ids, scores


def rbe_debug_scores_float(ix: Index, q, first_item: int, count: int, stream=None):
    qa, qap = _host(q, np.float32)
    if qa.shape != (ix.dim,):
        raise RbeError(RBE_EINVAL, f"expected q [{ix.dim}]")
    out = np.empty(count, dtype=np.float32)
    _check(load_library().rbe_debug_scores_float(ix.handle, qap, first_item, count, out.ctypes.data_as(_vp),
                                                 _stream_ptr(stream)))
    return out


def rbe_set_profiling(ix: Index, enabled: bool):
    _check(load_library().rbe_set_profiling(ix.handle, int(bool(enabled))))


def rbe_get_search_stats(ix: Index) -> dict:
    st = rbe_search_stats()
    _check(load_library().rbe_get_search_stats(ix.handle, ctypes.byref(st)))
    n = st.n_levels
    return {
        "n_levels": n, "fallback": st.fallback, "grid_blocks": st.grid_blocks, "deep_rows": st.deep_rows,
        "items_scanned": list(st.items_scanned)[:n], "candidates_max": list(st.candidates_max)[:n],
        "scan_ms": list(st.scan_ms)[:n], "select_ms": list(st.select_ms)[:n],
        "total_gpu_ms": st.total_gpu_ms, "deep_units": st.deep_units,
        "scan_kernel": [KERNEL_NAMES.get(v, str(v)) for v in list(st.scan_kernel)[:n]],
        "last_level_parts": st.last_level_parts, "deep_rows_level": list(st.deep_rows_level)[:n],
    }


def rbe_set_tuning(ix: Index, cand_capacity: int = 0, blocks_per_cu: int = 0):
    _check(load_library().rbe_set_tuning(ix.handle, cand_capacity, blocks_per_cu))


def rbe_debug_tile_to_phys(n_tiles: int, sample_ratio: int, tile: int) -> int:
    return int(load_library().rbe_debug_tile_to_phys(n_tiles, sample_ratio, tile))


def rbe_debug_phys_to_tile(n_tiles: int, sample_ratio: int, phys: int) -> int:
    return int(load_library().rbe_debug_phys_to_tile(n_tiles, sample_ratio, phys))


def rbe_debug_exact_plan(n_items: int, sample_ratio: int, cand_capacity: int, k: int):
    """Levels of the exact-mode plan as (first_tile, end_tile) physical ranges (host only)."""
    n = np.zeros(1, dtype=np.uint32)
    first = np.zeros(RBE_MAX_LEVELS, dtype=np.uint32)
    end = np.zeros(RBE_MAX_LEVELS, dtype=np.uint32)
    _check(load_library().rbe_debug_exact_plan(n_items, sample_ratio, cand_capacity, k, n.ctypes.data,
                                               first.ctypes.data, end.ctypes.data))
    return [(int(first[i]), int(end[i])) for i in range(int(n[0]))]


def rbe_debug_batch_operands(q_planes, q_scales, dim: int, n_planes: int, dyadic: bool, q_float=None):
    """Query operands of the matrix-core batch scan (host only): fp16 bit patterns
    [tile][plane copy][part][lane][8], unscale [Q], start [Q] and the filter margin (0 for a dyadic index).
    q_float [Q][dim] replaces the binary queries (general scales only)."""
    if q_float is not None:
        q_float = np.ascontiguousarray(q_float, dtype=np.float32)
        Q, Pq = q_float.shape[0], 0
    else:
        q_planes = np.ascontiguousarray(q_planes, dtype=np.uint64)
        Q, Pq = q_planes.shape[0], q_planes.shape[1]
    if q_scales is not None:
        q_scales = np.ascontiguousarray(q_scales, dtype=np.float32)
    cap = ((Q + 15) // 16) * 4 * (dim // 32) * 64 * 8
    halves = np.zeros(cap, dtype=np.uint16)
    unscale = np.zeros(Q, dtype=np.float32)
    start = np.zeros(Q, dtype=np.float32)
    shape = np.zeros(4, dtype=np.uint32)
    _check(load_library().rbe_debug_batch_operands(
        None if q_float is not None else q_planes.ctypes.data, None if q_scales is None else q_scales.ctypes.data,
        None if q_float is None else q_float.ctypes.data, Q, Pq, dim, n_planes,
        1 if dyadic else 0, halves.ctypes.data, cap, unscale.ctypes.data, start.ctypes.data, shape.ctypes.data))
    tiles, copies, parts = (int(x) for x in shape[:3])
    out = halves[:tiles * copies * parts * 64 * 8].reshape(tiles, copies, parts, 64, 8)
    return out, unscale, start, float(shape[3:4].view(np.float32)[0])


def rbe_debug_batch_operands_i8(q_planes, q_scales, dim: int, q_float=None):
    """Eight-bit integer query operands of the matrix-core batch scan (host only; general scales): int8
    [tile][part][lane][16], unscale [Q], start [Q], mass [Q] and the filter margin.  q_float [Q][dim] replaces
    the binary queries."""
    if q_float is not None:
        q_float = np.ascontiguousarray(q_float, dtype=np.float32)
        Q, Pq = q_float.shape[0], 0
    else:
        q_planes = np.ascontiguousarray(q_planes, dtype=np.uint64)
        q_scales = np.ascontiguousarray(q_scales, dtype=np.float32)
        Q, Pq = q_planes.shape[0], q_planes.shape[1]
    tiles, parts = (Q + 15) // 16, dim // 64
    ops = np.zeros((tiles, parts, 64, 16), dtype=np.int8)
    unscale, start, mass = (np.zeros(Q, dtype=np.float32) for _ in range(3))
    margin = np.zeros(1, dtype=np.float32)
    _check(load_library().rbe_debug_batch_operands_i8(
        None if q_float is not None else q_planes.ctypes.data, None if q_float is not None else q_scales.ctypes.data,
        None if q_float is None else q_float.ctypes.data, Q, Pq, dim, ops.ctypes.data, ops.nbytes,
        unscale.ctypes.data, start.ctypes.data, mass.ctypes.data, margin.ctypes.data))
    return ops, unscale, start, mass, float(margin[0])


def rbe_debug_batch_operands_i8_dyadic(q_planes, dim: int, n_item_planes: int):
    """Eight-bit integer query operands of the matrix-core batch scan on a dyadic index (host only): int8
    [tile][item plane][part][lane][16], unscale [Q], start [Q], mass [Q]."""
    q_planes = np.ascontiguousarray(q_planes, dtype=np.uint64)
    Q, Pq = q_planes.shape[0], q_planes.shape[1]
    tiles, parts = (Q + 15) // 16, dim // 64
    ops = np.zeros((tiles, n_item_planes, parts, 64, 16), dtype=np.int8)
    unscale, start, mass = (np.zeros(Q, dtype=np.float32) for _ in range(3))
    _check(load_library().rbe_debug_batch_operands_i8_dyadic(
        q_planes.ctypes.data, Q, Pq, dim, n_item_planes, ops.ctypes.data, ops.nbytes,
        unscale.ctypes.data, start.ctypes.data, mass.ctypes.data))
    return ops, unscale, start, mass


def rbe_debug_query_mass(q_planes, q_scales, dim: int, dyadic: bool = False):
    """Mass of one query ([Pq][W] planes, [Pq] scales) as the progressive scan uses it (host only):
    (x, y) floats for general scales, (h_min, 0) with h_min an int for a dyadic index."""
    q_planes = np.ascontiguousarray(q_planes, dtype=np.uint64)
    if q_scales is not None:
        q_scales = np.ascontiguousarray(q_scales, dtype=np.float32)
    out = np.zeros(2, dtype=np.float32)
    _check(load_library().rbe_debug_query_mass(q_planes.ctypes.data, None if q_scales is None else q_scales.ctypes.data,
                                               q_planes.shape[0], dim, 1 if dyadic else 0, out.ctypes.data))
    if dyadic:
        return int(out[:1].view(np.uint32)[0]), 0.0
    return float(out[0]), float(out[1])


def rbe_debug_set_plan_split(ix: Index, mode: int):
    """0 = automatic, 1 = never, 2 = always take the last level of an exact search in two parts."""
    _check(load_library().rbe_debug_set_plan_split(ix.handle, mode))


def rbe_debug_set_progressive(ix: Index, enabled):
    """False/0 = off, True/1 = on, 2 = on without the one-byte scale copies, 3 = on without the first stage on plane 0 alone."""
    _check(load_library().rbe_debug_set_progressive(ix.handle, int(enabled)))


def rbe_debug_set_nearlossless_path(ix: Index, path: int):
    """0 = exact scans + selection by groups (default), 1 = the per-thread-queue scan of Algorithm 1."""
    _check(load_library().rbe_debug_set_nearlossless_path(ix.handle, path))


def rbe_debug_set_batch_path(ix: Index, path: int):
    """0 = automatic, 1 = XOR/popcount kernel, 2 = matrix-core kernel, 3 = matrix-core kernel with half operands only."""
    _check(load_library().rbe_debug_set_batch_path(ix.handle, path))


def rbe_debug_popcounts(ix: Index, q_planes, first_item: int, count: int, stream=None):
    qp, qpp = _host(q_planes, np.uint64)
    Pq = qp.shape[0]
    out = np.empty((count, ix.n_planes, Pq), dtype=np.int32)
    _check(load_library().rbe_debug_popcounts(ix.handle, qpp, Pq, first_item, count, out.ctypes.data_as(_vp),
                                              _stream_ptr(stream)))
    return out


def rbe_debug_scores(ix: Index, q_planes, q_scales, first_item: int, count: int, stream=None):
    qp, qpp = _host(q_planes, np.uint64)
    qsp = None
    if q_scales is not None:
        qs, qsp = _host(q_scales, np.float32)
    out = np.empty(count, dtype=np.float32)
    _check(load_library().rbe_debug_scores(ix.handle, qpp, qsp, qp.shape[0], first_item, count,
                                           out.ctypes.data_as(_vp), _stream_ptr(stream)))
    return out


def rbe_debug_read_scales(ix: Index, first_item: int, count: int, stream=None):
    out = np.empty((ix.n_planes, count), dtype=np.float32)
    _check(load_library().rbe_debug_read_scales(ix.handle, first_item, count, out.ctypes.data_as(_vp),
                                                _stream_ptr(stream)))
    return out


def rbe_debug_read_planes(ix: Index, first_item: int, count: int, stream=None):
    out = np.empty((ix.n_planes, count, ix.dim // 64), dtype=np.uint64)
    _check(load_library().rbe_debug_read_planes(ix.handle, first_item, count, out.ctypes.data_as(_vp),
                                                _stream_ptr(stream)))
    return out


def rbe_debug_copy(dst, src, stream=None):
    """Plain device-to-device copy kernel between two torch cuda tensors of equal byte size."""
    nbytes = src.numel() * src.element_size()
    if nbytes != dst.numel() * dst.element_size() or not (src.is_cuda and dst.is_cuda):
        raise RbeError(RBE_EINVAL, "src and dst must be cuda tensors of equal byte size")
    _check(load_library().rbe_debug_copy(_vp(dst.data_ptr()), _vp(src.data_ptr()), nbytes, _stream_ptr(stream)))


def rbe_debug_read(src, sink, stream=None):
    """Read-only streaming kernel over a torch cuda tensor; `sink` is a cuda tensor of >= 8 MiB."""
    if not (src.is_cuda and sink.is_cuda):
        raise RbeError(RBE_EINVAL, "src and sink must be cuda tensors")
    _check(load_library().rbe_debug_read(_vp(src.data_ptr()), src.numel() * src.element_size(), _vp(sink.data_ptr()),
                                         sink.numel() * sink.element_size(), _stream_ptr(stream)))


def rbe_strerror(code: int) -> str:
    return load_library().rbe_strerror(code).decode()
