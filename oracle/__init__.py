"""ctypes binding of the C oracle (``comet_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, ``__graft_entry__.smoke()``
and the ``cpu_baseline`` leg of ``bench.py``.  The HIP library and its Python
binding never import this package, and this package never imports them.

All matrices are C-contiguous ``numpy.uint64`` arrays; arithmetic is mod 2^64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "comet_oracle.c")
_LIB = os.path.join(_HERE, "libcomet_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over output rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-std=c99", "-shared", "-fPIC",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        # every entry point with its C prototype, so that sizes travel at their declared width
        protos = {
            "co_encode": [vp, vp, sz, i], "co_decode": [vp, vp, sz, i],
            "co_share": [vp, vp, vp, vp, sz], "co_reconstruct": [vp, vp, vp, sz],
            "co_ring_matmul": [vp, vp, vp, i, i, i],
            "co_ring_matmul_rows": [vp, vp, vp, i, i, i, i, i],
            "co_mask_share": [vp, vp, vp, sz], "co_open": [vp, vp, vp, sz],
            "co_compact_mask": [vp, i, i, vp],
            "co_index_cols": [vp, i, i, vp, i, i, vp], "co_index_rows": [vp, i, i, vp, i, i, vp],
            "co_beaver_share": [i, vp, vp, vp, vp, vp, vp, vp, i, i, i],
            "co_beaver_share_rows": [i, vp, vp, vp, vp, vp, vp, vp, i, i, i, i, i],
            "co_beaver_share_at": [i, vp, vp, vp, vp, vp, i, i, i, i, i],
            "co_beaver_share_blocks": [i, vp, vp, vp, vp, vp, vp, vp, vp, i, i, i],
            "co_beaver_share_sparse_input": [i, vp, vp, vp, vp, vp, vp, vp, i, i, i],
            "co_permute_mask": [vp, vp, vp, vp, i, i, i, i],
            "co_scatter_cols": [vp, vp, i, i, vp, i, i],
            "co_truncate_share": [i, vp, vp, sz, i],
        }
        for name, args in protos.items():
            fn = getattr(_lib, name)
            fn.argtypes = args
            fn.restype = None
        _lib.co_compact_mask.restype = ctypes.c_int
        _lib.co_beaver_share_at.restype = ctypes.c_uint64
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _u64(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint64, a.dtype
    return a


def num_threads() -> int:
    """Threads the OpenMP loops will use (honours OMP_NUM_THREADS)."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        return int(env.split(",")[0])
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


# ---- fixed point ----

def encode(x: np.ndarray, frac_bits: int = 16) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    q = np.empty(x.shape, dtype=np.uint64)
    lib().co_encode(_p(x), _p(q), ctypes.c_size_t(x.size), ctypes.c_int(frac_bits))
    return q


def decode(q: np.ndarray, frac_bits: int = 16) -> np.ndarray:
    q = _u64(q)
    x = np.empty(q.shape, dtype=np.float64)
    lib().co_decode(_p(q), _p(x), ctypes.c_size_t(q.size), ctypes.c_int(frac_bits))
    return x


# ---- sharing ----

def share(v: np.ndarray, r: np.ndarray):
    v, r = _u64(v), _u64(r)
    assert v.shape == r.shape
    v0, v1 = np.empty_like(v), np.empty_like(v)
    lib().co_share(_p(v), _p(r), _p(v0), _p(v1), ctypes.c_size_t(v.size))
    return v0, v1


def reconstruct(v0: np.ndarray, v1: np.ndarray) -> np.ndarray:
    v0, v1 = _u64(v0), _u64(v1)
    assert v0.shape == v1.shape
    v = np.empty_like(v0)
    lib().co_reconstruct(_p(v0), _p(v1), _p(v), ctypes.c_size_t(v.size))
    return v


# ---- ring product ----

def ring_matmul(x: np.ndarray, y: np.ndarray) -> np.ndarray:
    x, y = _u64(x), _u64(y)
    m, k = x.shape
    k2, n = y.shape
    assert k == k2
    z = np.empty((m, n), dtype=np.uint64)
    lib().co_ring_matmul(_p(x), _p(y), _p(z), m, k, n)
    return z


# ---- masking / opening ----

def mask_share(x_i: np.ndarray, a_i: np.ndarray) -> np.ndarray:
    x_i, a_i = _u64(x_i), _u64(a_i)
    assert x_i.shape == a_i.shape
    d = np.empty_like(x_i)
    lib().co_mask_share(_p(x_i), _p(a_i), _p(d), ctypes.c_size_t(d.size))
    return d


def open_(d0: np.ndarray, d1: np.ndarray) -> np.ndarray:
    d0, d1 = _u64(d0), _u64(d1)
    assert d0.shape == d1.shape
    e = np.empty_like(d0)
    lib().co_open(_p(d0), _p(d1), _p(e), ctypes.c_size_t(e.size))
    return e


# ---- mask -> indices, indexing ----

def compact_mask(mask: np.ndarray) -> np.ndarray:
    """``mask``: uint8 ``[n_tok, nb]`` (or ``[nb]``).  Ascending active block ids."""
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    if mask.ndim == 1:
        mask = mask[None, :]
    n_tok, nb = mask.shape
    idx = np.empty(nb, dtype=np.int32)
    t = lib().co_compact_mask(_p(mask), n_tok, nb, _p(idx))
    return idx[:t].copy()


def index_cols(mat: np.ndarray, idx: np.ndarray, bs: int) -> np.ndarray:
    mat = _u64(mat)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    rows, cols = mat.shape
    out = np.empty((rows, len(idx) * bs), dtype=np.uint64)
    lib().co_index_cols(_p(mat), rows, cols, _p(idx), len(idx), bs, _p(out))
    return out


def index_rows(mat: np.ndarray, idx: np.ndarray, bs: int) -> np.ndarray:
    mat = _u64(mat)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    rows, cols = mat.shape
    out = np.empty((len(idx) * bs, cols), dtype=np.uint64)
    lib().co_index_rows(_p(mat), rows, cols, _p(idx), len(idx), bs, _p(out))
    return out


# ---- Eq. 1, matrix form ----

def beaver_share(party: int, e, f, a_i, b_i, c_i) -> np.ndarray:
    e, f, a_i, b_i, c_i = map(_u64, (e, f, a_i, b_i, c_i))
    m, k = e.shape
    k2, n = f.shape
    assert k == k2 and a_i.shape == (m, k) and b_i.shape == (k, n) and c_i.shape == (m, n)
    z = np.empty((m, n), dtype=np.uint64)
    tmp = np.empty((m, n), dtype=np.uint64)
    lib().co_beaver_share(party, _p(e), _p(f), _p(a_i), _p(b_i), _p(c_i), _p(z), _p(tmp), m, k, n)
    return z


def beaver_share_rows(party: int, e, f, a_i, b_i, c_i, r0: int, r1: int) -> np.ndarray:
    e, f, a_i, b_i, c_i = map(_u64, (e, f, a_i, b_i, c_i))
    m, k = e.shape
    k2, n = f.shape
    assert k == k2 and a_i.shape == (m, k) and b_i.shape == (k, n) and c_i.shape == (m, n)
    assert 0 <= r0 <= r1 <= m
    z = np.empty((r1 - r0, n), dtype=np.uint64)
    tmp = np.empty((r1 - r0, n), dtype=np.uint64)
    lib().co_beaver_share_rows(party, _p(e), _p(f), _p(a_i), _p(b_i), _p(c_i), _p(z), _p(tmp),
                               m, k, n, r0, r1)
    return z


def beaver_share_at(party: int, e, f, a_i, b_i, c_i, r: int, c: int) -> int:
    e, f, a_i, b_i, c_i = map(_u64, (e, f, a_i, b_i, c_i))
    m, k = e.shape
    n = f.shape[1]
    return int(lib().co_beaver_share_at(party, _p(e), _p(f), _p(a_i), _p(b_i), _p(c_i),
                                        m, k, n, r, c))


# ---- Protocols 2 and 3 in general form, one pass over all components / columns ----

def beaver_share_blocks(party: int, e, f, a_i, b_i, c_i, row_comp, col_comp) -> np.ndarray:
    """Protocol 2 merged: element (r, c) is computed iff ``row_comp[r] == col_comp[c] >= 0``."""
    e, f, a_i, b_i, c_i = map(_u64, (e, f, a_i, b_i, c_i))
    row_comp = np.ascontiguousarray(row_comp, dtype=np.int32)
    col_comp = np.ascontiguousarray(col_comp, dtype=np.int32)
    m, k = e.shape
    n = f.shape[1]
    assert f.shape == (k, n) and a_i.shape == (m, k) and b_i.shape == (k, n) and c_i.shape == (m, n)
    assert row_comp.shape == (m,) and col_comp.shape == (n,)
    z = np.empty((m, n), dtype=np.uint64)
    lib().co_beaver_share_blocks(party, _p(e), _p(f), _p(a_i), _p(b_i), _p(c_i), _p(row_comp),
                                 _p(col_comp), _p(z), m, k, n)
    return z


def beaver_share_sparse_input(party: int, e, f, a_i, b_i, c_i, s) -> np.ndarray:
    """Protocol 3 summed over its columns: entries of E / A_i outside ``s`` take no part."""
    e, f, a_i, b_i, c_i = map(_u64, (e, f, a_i, b_i, c_i))
    s = np.ascontiguousarray(s, dtype=np.uint8)
    m, k = e.shape
    n = f.shape[1]
    assert f.shape == (k, n) and a_i.shape == (m, k) and b_i.shape == (k, n) and c_i.shape == (m, n)
    assert s.shape == (m, k)
    z = np.empty((m, n), dtype=np.uint64)
    lib().co_beaver_share_sparse_input(party, _p(e), _p(f), _p(a_i), _p(b_i), _p(c_i), _p(s), _p(z),
                                       m, k, n)
    return z


# ---- oblivious shuffle steps, merge to full width, share-local rescaling ----

def permute_mask(src, perm, mask, axis: int, sign: int) -> np.ndarray:
    """dst = perm(src) +/- mask along columns (axis 0) or rows (axis 1); p(x)_j = x[p[j]]."""
    src, mask = _u64(src), _u64(mask)
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    rows, cols = src.shape
    assert mask.shape == src.shape and len(perm) == (cols if axis == 0 else rows)
    dst = np.empty_like(src)
    lib().co_permute_mask(_p(src), _p(perm), _p(mask), _p(dst), rows, cols, axis, sign)
    return dst


def scatter_cols(compact, idx, bs: int, n_full: int) -> np.ndarray:
    compact = _u64(compact)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    m = compact.shape[0]
    assert compact.shape[1] == len(idx) * bs
    full = np.empty((m, n_full), dtype=np.uint64)
    lib().co_scatter_cols(_p(compact), _p(idx), len(idx), bs, _p(full), m, n_full)
    return full


def truncate_share(party: int, z, frac_bits: int = 16) -> np.ndarray:
    z = _u64(z)
    out = np.empty_like(z)
    lib().co_truncate_share(party, _p(z), _p(out), z.size, frac_bits)
    return out
