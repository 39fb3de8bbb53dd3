"""ctypes front end of the CPU fp64 checker (slimspec_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The GPU package never imports this module and
this module never imports the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "slimspec_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_slimspec.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile slimspec_oracle.c with gcc (-O2, OpenMP) into liboracle_slimspec.so."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    # -ffp-contract=off / no fast-math: every fp64 operation is rounded as written.
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
           "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build(force=False)
    lib = ctypes.CDLL(_LIB)
    c_i, c_p = ctypes.c_int, ctypes.c_void_p
    lib.oracle_num_threads.restype = c_i
    lib.oracle_down_projection.argtypes = [c_p, c_p, c_i, c_i, c_i, c_p]
    lib.oracle_log_softmax_topk.argtypes = [c_p, c_i, c_i, c_p, c_p, c_p, c_p]
    lib.oracle_slimspec_head_topk.argtypes = [c_p, c_p, c_p, c_i, c_i, c_i, c_i, c_i,
                                              c_p, c_p, c_p, c_p, c_p]
    lib.oracle_full_head_topk.argtypes = [c_p, c_p, c_i, c_i, c_i, c_i, c_i,
                                          c_p, c_p, c_p, c_p, c_p]
    lib.oracle_slimspec_logits_at.argtypes = [c_p, c_p, c_p, c_i, c_i, c_i, c_i, c_p, c_p, c_i, c_p]
    lib.oracle_full_logits_at.argtypes = [c_p, c_p, c_i, c_i, c_i, c_i, c_p, c_p, c_i, c_p]
    c_u64 = ctypes.c_uint64
    lib.oracle_truncated_head_topk.argtypes = [c_p, c_p, c_i, c_p, c_i, c_i, c_i, c_i, c_p, c_p, c_p, c_p, c_p]
    lib.oracle_slimspec_head_topk_positions.argtypes = [c_p, c_p, c_p, c_i, c_p, c_i, c_i, c_i, c_i, c_i,
                                                        c_p, c_p, c_p, c_p, c_p]
    lib.oracle_gumbel_noise.argtypes = [c_u64, ctypes.c_int32, ctypes.c_int32]
    lib.oracle_gumbel_noise.restype = ctypes.c_double
    lib.oracle_sample_row.argtypes = [c_p, c_i, c_u64, ctypes.c_int32, c_p, c_p]
    lib.oracle_head_sample.argtypes = [c_p, c_p, c_p, c_i, c_i, c_i, c_i, c_i, c_i, c_u64,
                                       c_p, c_p, c_p, c_p, c_p, c_p]
    lib.oracle_routed_head_topk.argtypes = [c_p, c_p, c_p, c_p, c_i, c_i, c_i, c_i, c_i, c_i, c_i,
                                            c_p, c_p, c_p, c_p]
    for f in (lib.oracle_down_projection, lib.oracle_log_softmax_topk, lib.oracle_slimspec_head_topk,
              lib.oracle_full_head_topk, lib.oracle_slimspec_logits_at, lib.oracle_full_logits_at,
              lib.oracle_truncated_head_topk, lib.oracle_slimspec_head_topk_positions, lib.oracle_sample_row,
              lib.oracle_head_sample, lib.oracle_routed_head_topk):
        f.restype = c_i
    _lib = lib
    return lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("bf16 inputs must be uint16 bit patterns")
    return a


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def down_projection(h: np.ndarray, A: np.ndarray) -> np.ndarray:
    """t = h A in fp64; h [rows,d], A [d,r] as bf16 bits."""
    h, A = _u16(h), _u16(A)
    rows, d = h.shape
    d2, r = A.shape
    assert d == d2
    t = np.empty((rows, r), dtype=np.float64)
    st = _load().oracle_down_projection(_ptr(h), _ptr(A), rows, d, r, _ptr(t))
    if st != 0:
        raise RuntimeError(f"oracle_down_projection failed: {st}")
    return t


def log_softmax_topk(z: np.ndarray, k: int):
    """Exact top-k (logit desc, id asc) + log-probabilities of one fp64 logit row."""
    z = np.ascontiguousarray(z, dtype=np.float64)
    assert z.ndim == 1
    V = z.shape[0]
    ids = np.empty(k, dtype=np.int32)
    lp = np.empty(k, dtype=np.float32)
    lse = np.empty(1, dtype=np.float64)
    gap = np.empty(k, dtype=np.float64)
    st = _load().oracle_log_softmax_topk(_ptr(z), V, k, _ptr(ids), _ptr(lp), _ptr(lse), _ptr(gap))
    if st != 0:
        raise RuntimeError(f"oracle_log_softmax_topk failed: {st}")
    return ids, lp, float(lse[0]), gap


class HeadResult:
    __slots__ = ("ids", "logprobs", "lse", "gap", "z")

    def __init__(self, ids, logprobs, lse, gap, z):
        self.ids, self.logprobs, self.lse, self.gap, self.z = ids, logprobs, lse, gap, z


def slimspec_head_topk(h, A, B, k: int, return_logits: bool = False) -> HeadResult:
    """Low-rank head z = (h A) B reduced to top-k ids + natural-log probabilities (fp64 inside)."""
    h, A, B = _u16(h), _u16(A), _u16(B)
    rows, d = h.shape
    d2, r = A.shape
    r2, V = B.shape
    assert d == d2 and r == r2
    ids = np.empty((rows, k), dtype=np.int32)
    lp = np.empty((rows, k), dtype=np.float32)
    lse = np.empty(rows, dtype=np.float64)
    gap = np.empty((rows, k), dtype=np.float64)
    z = np.empty((rows, V), dtype=np.float64) if return_logits else None
    st = _load().oracle_slimspec_head_topk(_ptr(h), _ptr(A), _ptr(B), rows, d, r, V, k,
                                           _ptr(ids), _ptr(lp), _ptr(lse), _ptr(gap), _ptr(z))
    if st != 0:
        raise RuntimeError(f"oracle_slimspec_head_topk failed: {st}")
    return HeadResult(ids, lp, lse, gap, z)


def full_head_topk(h, W, k: int, return_logits: bool = False) -> HeadResult:
    """Full head z = h W (W bf16 bits or fp32) reduced to top-k ids + log-probabilities."""
    h = _u16(h)
    W = np.ascontiguousarray(W)
    if W.dtype == np.float32:
        w_is_f32 = 1
    elif W.dtype == np.uint16:
        w_is_f32 = 0
    else:
        raise TypeError("W must be uint16 (bf16 bits) or float32")
    rows, d = h.shape
    d2, V = W.shape
    assert d == d2
    ids = np.empty((rows, k), dtype=np.int32)
    lp = np.empty((rows, k), dtype=np.float32)
    lse = np.empty(rows, dtype=np.float64)
    gap = np.empty((rows, k), dtype=np.float64)
    z = np.empty((rows, V), dtype=np.float64) if return_logits else None
    st = _load().oracle_full_head_topk(_ptr(h), _ptr(W), w_is_f32, rows, d, V, k,
                                       _ptr(ids), _ptr(lp), _ptr(lse), _ptr(gap), _ptr(z))
    if st != 0:
        raise RuntimeError(f"oracle_full_head_topk failed: {st}")
    return HeadResult(ids, lp, lse, gap, z)


def slimspec_logits_at(h, A, B, row_idx, col_idx) -> np.ndarray:
    """fp64 logits of the low-rank head at the given (row, id) pairs only."""
    h, A, B = _u16(h), _u16(A), _u16(B)
    rows, d = h.shape
    r, V = B.shape
    ri = np.ascontiguousarray(row_idx, dtype=np.int32).ravel()
    ci = np.ascontiguousarray(col_idx, dtype=np.int32).ravel()
    assert ri.shape == ci.shape
    out = np.empty(ri.shape[0], dtype=np.float64)
    st = _load().oracle_slimspec_logits_at(_ptr(h), _ptr(A), _ptr(B), rows, d, r, V,
                                           _ptr(ri), _ptr(ci), ri.shape[0], _ptr(out))
    if st != 0:
        raise RuntimeError(f"oracle_slimspec_logits_at failed: {st}")
    return out


def full_logits_at(h, W, row_idx, col_idx) -> np.ndarray:
    """fp64 logits of the full head at the given (row, id) pairs only."""
    h = _u16(h)
    W = np.ascontiguousarray(W)
    w_is_f32 = 1 if W.dtype == np.float32 else 0
    if not w_is_f32 and W.dtype != np.uint16:
        raise TypeError("W must be uint16 (bf16 bits) or float32")
    rows, d = h.shape
    _, V = W.shape
    ri = np.ascontiguousarray(row_idx, dtype=np.int32).ravel()
    ci = np.ascontiguousarray(col_idx, dtype=np.int32).ravel()
    out = np.empty(ri.shape[0], dtype=np.float64)
    st = _load().oracle_full_logits_at(_ptr(h), _ptr(W), w_is_f32, rows, d, V,
                                       _ptr(ri), _ptr(ci), ri.shape[0], _ptr(out))
    if st != 0:
        raise RuntimeError(f"oracle_full_logits_at failed: {st}")
    return out


def _w_kind(W):
    W = np.ascontiguousarray(W)
    if W.dtype == np.float32:
        return W, 1
    if W.dtype == np.uint16:
        return W, 0
    raise TypeError("W must be uint16 (bf16 bits) or float32")


def truncated_head_topk(h, W_tr, id_map, k: int, return_logits: bool = False) -> HeadResult:
    """Full head over the kept columns W_tr [d, V_tr]; emitted ids are id_map[column] (ties: smaller column)."""
    h = _u16(h)
    W_tr, w_is_f32 = _w_kind(W_tr)
    id_map = np.ascontiguousarray(id_map, dtype=np.int32)
    rows, d = h.shape
    d2, V = W_tr.shape
    assert d == d2 and id_map.shape == (V,)
    ids = np.empty((rows, k), dtype=np.int32)
    lp = np.empty((rows, k), dtype=np.float32)
    lse = np.empty(rows, dtype=np.float64)
    gap = np.empty((rows, k), dtype=np.float64)
    z = np.empty((rows, V), dtype=np.float64) if return_logits else None
    st = _load().oracle_truncated_head_topk(_ptr(h), _ptr(W_tr), w_is_f32, _ptr(id_map), rows, d, V, k,
                                            _ptr(ids), _ptr(lp), _ptr(lse), _ptr(gap), _ptr(z))
    if st != 0:
        raise RuntimeError(f"oracle_truncated_head_topk failed: {st}")
    return HeadResult(ids, lp, lse, gap, z)


def slimspec_head_topk_positions(h, A_stack, pos_offsets, B, k: int, return_logits: bool = False) -> HeadResult:
    """Low-rank head with one down-projection per drafted position: rows [pos_offsets[p], pos_offsets[p+1]) use A_stack[p]."""
    h, A_stack, B = _u16(h), _u16(A_stack), _u16(B)
    rows, d = h.shape
    n_pos, d2, r = A_stack.shape
    r2, V = B.shape
    off = np.ascontiguousarray(pos_offsets, dtype=np.int32)
    assert d == d2 and r == r2 and off.shape == (n_pos + 1,)
    ids = np.empty((rows, k), dtype=np.int32)
    lp = np.empty((rows, k), dtype=np.float32)
    lse = np.empty(rows, dtype=np.float64)
    gap = np.empty((rows, k), dtype=np.float64)
    z = np.empty((rows, V), dtype=np.float64) if return_logits else None
    st = _load().oracle_slimspec_head_topk_positions(_ptr(h), _ptr(A_stack), _ptr(off), n_pos, _ptr(B), rows, d, r, V, k,
                                                     _ptr(ids), _ptr(lp), _ptr(lse), _ptr(gap), _ptr(z))
    if st != 0:
        raise RuntimeError(f"oracle_slimspec_head_topk_positions failed: {st}")
    return HeadResult(ids, lp, lse, gap, z)


def gumbel_noise(seed: int, row: int, ids) -> np.ndarray:
    """The standard Gumbel draws g(seed, row, id) that the sampling outputs use, as fp64."""
    lib = _load()
    return np.array([lib.oracle_gumbel_noise(seed, row, int(v)) for v in np.asarray(ids).ravel()], dtype=np.float64)


def sample_row(z, seed: int, row: int):
    """One draw from softmax(z): (id, z[id] + g[id]) of the largest z_v + g_v."""
    z = np.ascontiguousarray(z, dtype=np.float64)
    out_id = np.empty(1, dtype=np.int32)
    best = np.empty(1, dtype=np.float64)
    st = _load().oracle_sample_row(_ptr(z), z.shape[0], seed, row, _ptr(out_id), _ptr(best))
    if st != 0:
        raise RuntimeError(f"oracle_sample_row failed: {st}")
    return int(out_id[0]), float(best[0])


class SampleResult:
    __slots__ = ("ids", "logprobs", "lse", "sample_ids", "sample_logprobs", "z")

    def __init__(self, ids, logprobs, lse, sample_ids, sample_logprobs, z):
        self.ids, self.logprobs, self.lse = ids, logprobs, lse
        self.sample_ids, self.sample_logprobs, self.z = sample_ids, sample_logprobs, z


def head_sample(h, A, M, k: int, seed: int, return_logits: bool = False) -> SampleResult:
    """Top-k, lse and one Gumbel-max sample per row; A is None for the full head (then M is W)."""
    h = _u16(h)
    rows, d = h.shape
    if A is not None:
        A, M = _u16(A), _u16(M)
        r, m_is_f32 = A.shape[1], 0
    else:
        M, m_is_f32 = _w_kind(M)
        r = 0
    V = M.shape[1]
    ids = np.empty((rows, k), dtype=np.int32)
    lp = np.empty((rows, k), dtype=np.float32)
    lse = np.empty(rows, dtype=np.float64)
    sid = np.empty(rows, dtype=np.int32)
    slp = np.empty(rows, dtype=np.float32)
    z = np.empty((rows, V), dtype=np.float64) if return_logits else None
    st = _load().oracle_head_sample(_ptr(h), _ptr(A), _ptr(M), m_is_f32, rows, d, r, V, k, seed,
                                    _ptr(ids), _ptr(lp), _ptr(lse), _ptr(sid), _ptr(slp), _ptr(z))
    if st != 0:
        raise RuntimeError(f"oracle_head_sample failed: {st}")
    return SampleResult(ids, lp, lse, sid, slp, z)


def routed_head_topk(h, A, B, W, k_route: int, k: int):
    """Router-then-exact head: (ids [rows,k], logprobs over the routed subset, lse of the subset, route_ids [rows,k_route])."""
    h, A, B = _u16(h), _u16(A), _u16(B)
    W, w_is_f32 = _w_kind(W)
    rows, d = h.shape
    r, V = B.shape
    ids = np.empty((rows, k), dtype=np.int32)
    lp = np.empty((rows, k), dtype=np.float32)
    lse = np.empty(rows, dtype=np.float64)
    route = np.empty((rows, k_route), dtype=np.int32)
    st = _load().oracle_routed_head_topk(_ptr(h), _ptr(A), _ptr(B), _ptr(W), w_is_f32, rows, d, r, V, k_route, k,
                                         _ptr(ids), _ptr(lp), _ptr(lse), _ptr(route))
    if st != 0:
        raise RuntimeError(f"oracle_routed_head_topk failed: {st}")
    return ids, lp, lse, route
