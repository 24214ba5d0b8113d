"""CPU oracle for RBE retrieval -- TEST INFRASTRUCTURE ONLY.

A plain, slow, single-threaded reference of what the GPU library computes:
the stand-in encoder, the binary-dot-product score (Eq. 14 with the bit-wise
identity of Sec. 5.1), exact top-k, the near-lossless selector of Algorithm 1
(Sec. 6.2) and the miss-probability model of Appendix A.

It shares nothing with the GPU library (no code, header, table or helper) and
neither imports the other.  Only the tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package.

Parity status: every function here is pinned by CPU tests to something other
than itself (brute-force float dot products of unpacked vectors, closed forms,
invariants, the values printed in Table 7) except ``encode`` as a model of the
paper's *learned* RBE layers: the trained matrices of Eq. 8-11 are not
available, so the greedy binariser is pinned only to its own least-squares /
energy identities -- "parity unpinned" with respect to the paper's encoder.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

from .missprob import (expected_recall, miss_probability,  # noqa: F401
                       prob_threads_hit)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rbe_oracle.c")
_LIB = os.path.join(_HERE, "librbe_oracle.so")


def build(force: bool = False) -> str:
    """Compile the C part of the oracle with gcc (host only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-Wall", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _c():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u64, u32, i64 = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int64
        vp = ctypes.c_void_p
        lib.orc_binary_dot.restype = ctypes.c_int32
        lib.orc_binary_dot.argtypes = [vp, vp, u32]
        lib.orc_popcounts.restype = None
        lib.orc_popcounts.argtypes = [vp, u64, u32, u32, vp, u32, vp]
        lib.orc_scores.restype = None
        lib.orc_scores.argtypes = [vp, vp, u64, u32, u32, vp, vp, u32, u64, u64, vp]
        lib.orc_scores_at.restype = None
        lib.orc_scores_at.argtypes = [vp, vp, u64, u32, u32, vp, vp, u32, vp, u64, vp]
        lib.orc_topk.restype = i64
        lib.orc_topk.argtypes = [vp, vp, u64, u32, u32, vp, vp, u32, u64, u64, u64, vp, vp]
        lib.orc_topk_of_scores.restype = i64
        lib.orc_topk_of_scores.argtypes = [vp, vp, u64, u64, vp, vp]
        lib.orc_n_groups.restype = u64
        lib.orc_n_groups.argtypes = [u64, u64, u64]
        lib.orc_nearlossless.restype = i64
        lib.orc_nearlossless.argtypes = [vp, vp, u64, u32, u32, vp, vp, u32, u64, u64, u64, u64, vp, vp, vp, vp]
        lib.orc_encode.restype = None
        lib.orc_encode.argtypes = [vp, u64, u32, u32, vp, vp]
        lib.orc_scores_fq.restype = None
        lib.orc_scores_fq.argtypes = [vp, vp, u64, u32, u32, vp, u64, u64, vp]
        lib.orc_scores_at_fq.restype = None
        lib.orc_scores_at_fq.argtypes = [vp, vp, u64, u32, u32, vp, vp, u64, vp]
        lib.orc_topk_fq.restype = i64
        lib.orc_topk_fq.argtypes = [vp, vp, u64, u32, u32, vp, u64, u64, u64, vp, vp]
        lib.orc_recon_norms.restype = None
        lib.orc_recon_norms.argtypes = [vp, vp, u64, u32, u32, vp]
        _lib = lib
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _corpus(planes, scales):
    planes = np.ascontiguousarray(planes, dtype=np.uint64)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    if planes.ndim != 3 or scales.ndim != 2:
        raise ValueError("planes must be [P][N][W], scales [P][N]")
    P, N, W = planes.shape
    if scales.shape != (P, N):
        raise ValueError("scales shape does not match planes")
    return planes, scales, P, N, W


def _query(q_planes, q_scales, W):
    q_planes = np.ascontiguousarray(q_planes, dtype=np.uint64)
    q_scales = np.ascontiguousarray(q_scales, dtype=np.float32)
    if q_planes.ndim != 2 or q_planes.shape[1] != W or q_scales.shape != (q_planes.shape[0],):
        raise ValueError("query must be q_planes [Pq][W], q_scales [Pq]")
    return q_planes, q_scales, q_planes.shape[0]


def binary_dot(x_words, y_words) -> int:
    """x . y for x, y in {-1,+1}^d given as packed words (Sec. 5.1 identity)."""
    x = np.ascontiguousarray(x_words, dtype=np.uint64).ravel()
    y = np.ascontiguousarray(y_words, dtype=np.uint64).ravel()
    assert x.shape == y.shape
    return int(_c().orc_binary_dot(_p(x), _p(y), 64 * x.size))


def encode(x, n_planes: int):
    """Stand-in encoder: x [n][d] fp32 -> planes [P][n][W] u64, scales [P][n] f32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if x.ndim == 1:
        x = x[None, :]
    n, d = x.shape
    if d % 64:
        raise ValueError("d must be a multiple of 64")
    planes = np.zeros((n_planes, n, d // 64), dtype=np.uint64)
    scales = np.zeros((n_planes, n), dtype=np.float32)
    _c().orc_encode(_p(x), n, d, n_planes, _p(planes), _p(scales))
    return planes, scales


def popcounts(planes, q_planes):
    """popcount(Q_i XOR K_j[z]) as int32 [N][P][Pq]."""
    planes = np.ascontiguousarray(planes, dtype=np.uint64)
    P, N, W = planes.shape
    q_planes = np.ascontiguousarray(q_planes, dtype=np.uint64)
    Pq = q_planes.shape[0]
    out = np.zeros((N, P, Pq), dtype=np.int32)
    _c().orc_popcounts(_p(planes), N, 64 * W, P, _p(q_planes), Pq, _p(out))
    return out


def scores(planes, scales, q_planes, q_scales, z0: int = 0, z1: int | None = None):
    """Dense float64 scores of one query against items [z0, z1)."""
    planes, scales, P, N, W = _corpus(planes, scales)
    q_planes, q_scales, Pq = _query(q_planes, q_scales, W)
    z1 = N if z1 is None else z1
    out = np.zeros(z1 - z0, dtype=np.float64)
    _c().orc_scores(_p(planes), _p(scales), N, 64 * W, P, _p(q_planes), _p(q_scales), Pq, z0, z1, _p(out))
    return out


def scores_at(planes, scales, q_planes, q_scales, ids):
    """Float64 scores of one query against the listed item ids."""
    planes, scales, P, N, W = _corpus(planes, scales)
    q_planes, q_scales, Pq = _query(q_planes, q_scales, W)
    ids = np.ascontiguousarray(ids, dtype=np.int64)
    if ids.size and (ids.min() < 0 or ids.max() >= N):
        raise ValueError("id out of range")
    out = np.zeros(ids.size, dtype=np.float64)
    _c().orc_scores_at(_p(planes), _p(scales), N, 64 * W, P, _p(q_planes), _p(q_scales), Pq, _p(ids), ids.size, _p(out))
    return out


def topk(planes, scales, q_planes, q_scales, k: int, z0: int = 0, z1: int | None = None):
    """Exact top-k (score desc, id asc) of one query.  Returns (ids i64[k], scores f64[k])."""
    planes, scales, P, N, W = _corpus(planes, scales)
    q_planes, q_scales, Pq = _query(q_planes, q_scales, W)
    z1 = N if z1 is None else z1
    ids = np.zeros(k, dtype=np.int64)
    sc = np.zeros(k, dtype=np.float64)
    r = _c().orc_topk(_p(planes), _p(scales), N, 64 * W, P, _p(q_planes), _p(q_scales), Pq, z0, z1, k, _p(ids), _p(sc))
    if r < 0:
        raise MemoryError
    return ids, sc


def topk_of_scores(sc, ids, k: int):
    """Exact top-k of explicit (score, id) pairs; ids=None means 0..n-1."""
    sc = np.ascontiguousarray(sc, dtype=np.float64)
    if ids is not None:
        ids = np.ascontiguousarray(ids, dtype=np.int64)
    out_i = np.zeros(k, dtype=np.int64)
    out_s = np.zeros(k, dtype=np.float64)
    r = _c().orc_topk_of_scores(_p(sc), _p(ids) if ids is not None else None, sc.size, k, _p(out_i), _p(out_s))
    if r < 0:
        raise MemoryError
    return out_i, out_s


def n_groups(N: int, I: int, Tb: int = 256) -> int:
    return int(_c().orc_n_groups(N, Tb, I))


def nearlossless(planes, scales, q_planes, q_scales, k: int, I: int = 256, Tb: int = 256,
                 return_winners: bool = False, queue_len: int = 1):
    """Near-lossless selection (Algorithm 1, Sec. 6.2): ids z with equal
    (z div (Tb*I)) * Tb + z mod Tb form a group, every group forwards its best `queue_len`
    items (the paper's choice is 1), and the result is the exact top-k of what was forwarded.
    With return_winners the forwarded items come back as [n_groups, queue_len] arrays
    (squeezed for length 1)."""
    planes, scales, P, N, W = _corpus(planes, scales)
    q_planes, q_scales, Pq = _query(q_planes, q_scales, W)
    if queue_len < 1:
        raise ValueError("queue_len must be >= 1")
    ids = np.zeros(k, dtype=np.int64)
    sc = np.zeros(k, dtype=np.float64)
    G = n_groups(N, I, Tb)
    w_ids = np.zeros((G, queue_len), dtype=np.int64)
    w_sc = np.zeros((G, queue_len), dtype=np.float64)
    r = _c().orc_nearlossless(_p(planes), _p(scales), N, 64 * W, P, _p(q_planes), _p(q_scales), Pq,
                              Tb, I, queue_len, k, _p(ids), _p(sc), _p(w_ids), _p(w_sc))
    if r < 0:
        raise MemoryError
    if return_winners:
        if queue_len == 1:
            return ids, sc, w_ids[:, 0], w_sc[:, 0]
        return ids, sc, w_ids, w_sc
    return ids, sc


def recon_norms(planes, scales):
    """||sum_j a_j[z] b_z^j||_2 per item, float64 [N]."""
    planes, scales, P, N, W = _corpus(planes, scales)
    out = np.zeros(N, dtype=np.float64)
    _c().orc_recon_norms(_p(planes), _p(scales), N, 64 * W, P, _p(out))
    return out


def fold_cosine(planes, scales):
    """Per-item scales divided by the item's reconstructed norm (Sec. 5.1:
    the keyword-side magnitude is precomputed and stored with the embedding)."""
    nrm = recon_norms(planes, scales)
    safe = np.where(nrm > 0, nrm, 1.0)
    return (np.asarray(scales, dtype=np.float64) / safe[None, :]).astype(np.float32)


def _fquery(q, d):
    q = np.ascontiguousarray(q, dtype=np.float32)
    if q.shape != (d,):
        raise ValueError(f"float query must have shape ({d},)")
    return q


def scores_fq(planes, scales, q, z0: int = 0, z1: int | None = None):
    """Hybrid scoring (fp32 query x RBE items, the paper's model m_5): float64 scores of items [z0, z1)."""
    planes, scales, P, N, W = _corpus(planes, scales)
    q = _fquery(q, 64 * W)
    z1 = N if z1 is None else z1
    out = np.zeros(z1 - z0, dtype=np.float64)
    _c().orc_scores_fq(_p(planes), _p(scales), N, 64 * W, P, _p(q), z0, z1, _p(out))
    return out


def scores_at_fq(planes, scales, q, ids):
    planes, scales, P, N, W = _corpus(planes, scales)
    q = _fquery(q, 64 * W)
    ids = np.ascontiguousarray(ids, dtype=np.int64)
    if ids.size and (ids.min() < 0 or ids.max() >= N):
        raise ValueError("id out of range")
    out = np.zeros(ids.size, dtype=np.float64)
    _c().orc_scores_at_fq(_p(planes), _p(scales), N, 64 * W, P, _p(q), _p(ids), ids.size, _p(out))
    return out


def topk_fq(planes, scales, q, k: int, z0: int = 0, z1: int | None = None):
    planes, scales, P, N, W = _corpus(planes, scales)
    q = _fquery(q, 64 * W)
    z1 = N if z1 is None else z1
    ids = np.zeros(k, dtype=np.int64)
    sc = np.zeros(k, dtype=np.float64)
    r = _c().orc_topk_fq(_p(planes), _p(scales), N, 64 * W, P, _p(q), z0, z1, k, _p(ids), _p(sc))
    if r < 0:
        raise MemoryError
    return ids, sc


def recall(result_ids, exact_ids) -> float:
    """|result ∩ exact| / |exact|, ignoring -1 padding."""
    e = set(int(i) for i in exact_ids if i >= 0)
    if not e:
        return 1.0
    r = set(int(i) for i in result_ids if i >= 0)
    return len(e & r) / len(e)
