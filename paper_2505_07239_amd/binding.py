"""Thin ctypes binding of ``libcomet_ring.so`` (see ``include/comet_ring.h``).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  Tensors are ``torch.int64`` CUDA(-HIP) tensors whose bits are the
ring elements mod 2^64; torch is used for device memory and streams, nothing
else.  There is no CPU fallback: if the library is missing or a call fails, an
exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcomet_ring.so")

AXIS_COLS, AXIS_ROWS = 0, 1
OP_COMPACT, OP_SOMM, OP_SIMM = 0, 1, 2
FULL_A, FULL_B, WEIGHTS_NEURON_MAJOR, WEIGHT_PLANES = 1, 2, 4, 8
TUNE_GEMM_GRID, TUNE_GEMM_CHUNK, TUNE_GEMM_TILE, TUNE_SKINNY, TUNE_SKINNY_SLICES, TUNE_COMPONENTS = 0, 1, 2, 3, 4, 5
TUNE_TIMING_STRIDE, TUNE_GROUP = 6, 7

EXPORTS = [
    "comet_create", "comet_destroy", "comet_set_stream", "comet_last_error", "comet_version",
    "comet_workspace_bytes", "comet_mask_share", "comet_mask_share_gather", "comet_open",
    "comet_weight_planes_bytes", "comet_open_weight_planes", "comet_open_weight_planes_neuron_major",
    "comet_compact_mask", "comet_somm_share", "comet_somm_share_static", "comet_simm_share", "comet_share_group",
    "comet_somm_share_unopened", "comet_simm_share_unopened",
    "comet_components", "comet_somm_share_blocks", "comet_simm_share_masked",
    "comet_permute_mask", "comet_scatter_cols", "comet_truncate_share",
    "comet_set_tuning", "comet_timing_begin", "comet_timing_end", "comet_probe_mfma_i8", "comet_probe_valu_mac64", "comet_probe_copy",
]

_lib = None


class CometError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("comet_ring error %d: %s" % (code, msg))
        self.code = code


def load_library() -> ctypes.CDLL:
    """dlopen the in-tree library (build it first with ``paper_2505_07239_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s not found: run `python -m paper_2505_07239_amd.build` (needs hipcc)" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
    lib.comet_create.argtypes = [ctypes.POINTER(vp), i32]
    lib.comet_destroy.argtypes = [vp]
    lib.comet_set_stream.argtypes = [vp, vp]
    lib.comet_last_error.argtypes = [vp]
    lib.comet_last_error.restype = ctypes.c_char_p
    lib.comet_version.restype = ctypes.c_char_p
    lib.comet_workspace_bytes.argtypes = [i32, i64, i64, i64, i32]
    lib.comet_workspace_bytes.restype = sz
    lib.comet_mask_share.argtypes = [vp, vp, vp, vp, sz]
    lib.comet_open.argtypes = [vp, vp, vp, vp, sz]
    lib.comet_weight_planes_bytes.argtypes = [i64, i64]
    lib.comet_weight_planes_bytes.restype = sz
    lib.comet_open_weight_planes.argtypes = [vp, vp, vp, i64, i64, vp]
    lib.comet_open_weight_planes_neuron_major.argtypes = [vp, vp, vp, i64, i64, vp]
    lib.comet_mask_share_gather.argtypes = [vp, vp, vp, vp, i64, i64, i32, i32, vp, vp, i32]
    lib.comet_compact_mask.argtypes = [vp, vp, i64, i64, vp, vp, vp, sz]
    share = [vp, i32, i64, i64, i64, i32, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, sz]
    lib.comet_somm_share.argtypes = share
    lib.comet_simm_share.argtypes = share
    lib.comet_somm_share_static.argtypes = share[:-2]
    # (E, G_0, G_1, A_i, B_i, C_i, Z_i): one pointer more than the opened form
    lib.comet_somm_share_unopened.argtypes = share[:10] + [vp] + share[10:]
    lib.comet_simm_share_unopened.argtypes = share[:10] + [vp] + share[10:]
    lib.comet_share_group.argtypes = [vp, i32, i32, ctypes.POINTER(ShareOperands), i64, i64, i64, i32, vp, vp, i32,
                                      i32, vp, sz]
    lib.comet_components.argtypes = [vp, vp, i64, i64, vp, vp, vp, vp, vp, vp, vp]
    lib.comet_somm_share_blocks.argtypes = [vp, i32, i64, i64, i64, i32, vp, vp, vp, i32, vp, vp, i32,
                                            vp, vp, vp, vp, vp, vp, vp, sz]
    lib.comet_simm_share_masked.argtypes = [vp, i32, i64, i64, i64, i32, vp, vp, i32, i32, vp, i64,
                                            vp, vp, vp, vp, vp, vp, vp, sz]
    lib.comet_permute_mask.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, i32]
    lib.comet_scatter_cols.argtypes = [vp, vp, i64, i32, vp, vp, i32, vp, i64]
    lib.comet_truncate_share.argtypes = [vp, i32, vp, vp, sz, i32]
    lib.comet_probe_mfma_i8.argtypes = [vp, i32, i32, i32, vp, ctypes.POINTER(ctypes.c_double)]
    lib.comet_probe_valu_mac64.argtypes = [vp, i32, i32, vp, ctypes.POINTER(ctypes.c_double)]
    lib.comet_probe_copy.argtypes = [vp, vp, vp, sz]
    lib.comet_set_tuning.argtypes = [vp, i32, i32]
    lib.comet_timing_begin.argtypes = [vp, i32]
    lib.comet_timing_end.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int)]
    _lib = lib
    return lib


def workspace_bytes(op: int, m: int, k: int, n: int, bs: int) -> int:
    return int(load_library().comet_workspace_bytes(op, m, k, n, bs))


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _words(t: torch.Tensor, what: str) -> torch.Tensor:
    if t.dtype != torch.int64 or not t.is_cuda or not t.is_contiguous():
        raise TypeError("%s must be a contiguous int64 tensor on the GPU" % what)
    return t


SHARE_GROUP_MAX = 8


class ShareOperands(ctypes.Structure):
    """``comet_share_operands``: one member of a grouped share call."""
    _fields_ = [("party", ctypes.c_int32), ("reserved", ctypes.c_int32), ("E", ctypes.c_void_p),
                ("F", ctypes.c_void_p), ("A_i", ctypes.c_void_p), ("B_i", ctypes.c_void_p),
                ("C_i", ctypes.c_void_p), ("Z_i", ctypes.c_void_p)]


class WeightPlanes:
    """A weight-side operand (F or B_i) in the digit-plane format of ``comet_open_weight_planes``:
    the raw buffer plus the logical shape ``k x n`` of the matrix it stands for."""

    def __init__(self, buf: torch.Tensor, k: int, n: int):
        self.buf, self.shape = buf, (k, n)

    def data_ptr(self):
        return self.buf.data_ptr()


def _weights(t, what: str):
    """A weight-side operand: words (int64 tensor) or planes."""
    if isinstance(t, WeightPlanes):
        return t
    return _words(t, what)


def _operands(e, f, a_i, b_i, c_i) -> int:
    """Type checks of the five operands of a share call; returns the flag bit for weight planes
    (F and B_i are either both words or both planes)."""
    _words(e, "E"), _words(a_i, "A_i"), _words(c_i, "C_i")
    _weights(f, "F"), _weights(b_i, "B_i")
    if isinstance(f, WeightPlanes) != isinstance(b_i, WeightPlanes):
        raise TypeError("F and B_i must both be words or both be weight planes")
    return WEIGHT_PLANES if isinstance(f, WeightPlanes) else 0


def _index_list(blk_idx, n_blk_dev, n_blk_cap: int, required: bool):
    """The block list of a share / masking call: int32 on the GPU, at least n_blk_cap entries."""
    if n_blk_cap < 0:
        raise ValueError("n_blk_cap must not be negative")
    if blk_idx is None:
        if required:
            raise ValueError("blk_idx is required when an operand is indexed inside the kernel")
    else:
        if blk_idx.dtype != torch.int32 or not blk_idx.is_cuda or not blk_idx.is_contiguous():
            raise TypeError("blk_idx must be a contiguous int32 tensor on the GPU")
        # with the count on the device only its first *n_blk_dev entries are read
        if n_blk_dev is None and blk_idx.numel() < n_blk_cap:
            raise ValueError("blk_idx holds %d entries, n_blk_cap is %d" % (blk_idx.numel(), n_blk_cap))
    if n_blk_dev is not None:
        if n_blk_dev.dtype != torch.int32 or not n_blk_dev.is_cuda or n_blk_dev.numel() < 1:
            raise TypeError("n_blk_dev must be an int32 tensor on the GPU")


def _shape(t: torch.Tensor, shape, what: str):
    if tuple(t.shape) != tuple(shape):
        raise ValueError("%s has shape %s, expected %s" % (what, tuple(t.shape), tuple(shape)))


class Context:
    """One library context on one device; calls run on torch's current stream."""

    def __init__(self, device: int = 0):
        self.lib = load_library()
        self.device = device
        h = ctypes.c_void_p()
        rc = self.lib.comet_create(ctypes.byref(h), device)
        if rc != 0:
            raise CometError(rc, "comet_create failed (is device %d an MI355X?)" % device)
        self.h = h
        self._ws = None

    def close(self):
        if getattr(self, "h", None):
            self.lib.comet_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != 0:
            raise CometError(rc, self.lib.comet_last_error(self.h).decode())

    def _sync_stream(self):
        s = torch.cuda.current_stream(self.device).cuda_stream
        self._check(self.lib.comet_set_stream(self.h, ctypes.c_void_p(s)))

    def workspace(self, nbytes: int) -> Optional[torch.Tensor]:
        """A cached device buffer of at least ``nbytes`` (torch allocation, 256-byte aligned)."""
        if nbytes == 0:
            return None
        if self._ws is None or self._ws.numel() < nbytes:
            self._ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda:%d" % self.device)
        return self._ws

    # ---- (1) mask / open ----
    def mask_share(self, x_i, a_i, out=None):
        _words(x_i, "x_i"), _words(a_i, "a_i")
        out = torch.empty_like(x_i) if out is None else _words(out, "out")
        if a_i.numel() != x_i.numel() or out.numel() != x_i.numel():
            raise ValueError("x_i, a_i and out must hold the same number of words")
        self._sync_stream()
        self._check(self.lib.comet_mask_share(self.h, _ptr(x_i), _ptr(a_i), _ptr(out), x_i.numel()))
        return out

    def open(self, d_0, d_1, out=None):
        _words(d_0, "d_0"), _words(d_1, "d_1")
        out = torch.empty_like(d_0) if out is None else _words(out, "out")
        if d_1.numel() != d_0.numel() or out.numel() != d_0.numel():
            raise ValueError("d_0, d_1 and out must hold the same number of words")
        self._sync_stream()
        self._check(self.lib.comet_open(self.h, _ptr(d_0), _ptr(d_1), _ptr(out), d_0.numel()))
        return out

    def open_weight_planes(self, g_0, g_1=None, out=None, neuron_major=False) -> WeightPlanes:
        """F = g_0 + g_1 (or g_0 alone: offline packing of a triple share) as digit planes.
        ``neuron_major``: the operands are stored one row per column of the matrix (n x k)."""
        _words(g_0, "g_0")
        k, n = (g_0.shape[1], g_0.shape[0]) if neuron_major else g_0.shape
        if g_1 is not None:
            _words(g_1, "g_1")
            _shape(g_1, tuple(g_0.shape), "g_1")
        need = int(self.lib.comet_weight_planes_bytes(k, n))
        if out is None:
            out = torch.empty(max(need, 16), dtype=torch.uint8, device=g_0.device)
        elif out.dtype != torch.uint8 or not out.is_cuda or out.numel() < need:
            raise TypeError("out must be a uint8 tensor on the GPU of at least %d bytes" % need)
        self._sync_stream()
        call = self.lib.comet_open_weight_planes_neuron_major if neuron_major else self.lib.comet_open_weight_planes
        self._check(call(self.h, _ptr(g_0), _ptr(g_1), k, n, _ptr(out)))
        return WeightPlanes(out, k, n)

    def mask_share_gather(self, w_i, b_i, axis, bs, blk_idx, n_blk_dev, n_blk_cap, out=None):
        _words(w_i, "w_i"), _words(b_i, "b_i")
        rows, cols = w_i.shape
        ld = n_blk_cap * bs
        shape = (rows, ld) if axis == AXIS_COLS else (ld, cols)
        out = torch.empty(shape, dtype=torch.int64, device=w_i.device) if out is None else _words(out, "out")
        _shape(b_i, (rows, cols), "b_i"), _shape(out, shape, "out")
        _index_list(blk_idx, n_blk_dev, n_blk_cap, True)
        self._sync_stream()
        self._check(self.lib.comet_mask_share_gather(self.h, _ptr(w_i), _ptr(b_i), _ptr(out), rows,
                                                     cols, axis, bs, _ptr(blk_idx), _ptr(n_blk_dev),
                                                     n_blk_cap))
        return out

    # ---- (2) compact ----
    def compact_mask(self, mask, blk_idx=None, n_blk_dev=None):
        if mask.dtype != torch.uint8 or not mask.is_cuda or not mask.is_contiguous():
            raise TypeError("mask must be a contiguous uint8 tensor on the GPU")
        if mask.dim() == 1:
            mask = mask[None, :]
        n_tok, nb = mask.shape
        if blk_idx is None:
            blk_idx = torch.empty(max(nb, 1), dtype=torch.int32, device=mask.device)
        if n_blk_dev is None:
            n_blk_dev = torch.empty(1, dtype=torch.int32, device=mask.device)
        need = workspace_bytes(OP_COMPACT, n_tok, 0, nb, 0)
        ws = self.workspace(need)
        self._sync_stream()
        self._check(self.lib.comet_compact_mask(self.h, _ptr(mask), n_tok, nb, _ptr(blk_idx),
                                                _ptr(n_blk_dev), _ptr(ws), need))
        return blk_idx, n_blk_dev

    # ---- (3) output share ----
    def somm_share(self, party, bs, blk_idx, n_blk_dev, n_blk_cap, e, f, a_i, b_i, c_i,
                   b_full=True, neuron_major=False, out=None):
        """``neuron_major``: ``f`` and ``b_i`` are stored one row per neuron (n x k)."""
        planes = _operands(e, f, a_i, b_i, c_i)
        m, k = e.shape
        n_full = b_i.shape[0 if neuron_major else 1] if b_full else 0
        ld = n_blk_cap * bs
        out = torch.empty((m, ld), dtype=torch.int64, device=e.device) if out is None else _words(out, "out")
        self._somm_shapes(m, k, ld, n_full, f, a_i, b_i, c_i, out, b_full, neuron_major)
        _index_list(blk_idx, n_blk_dev, n_blk_cap, b_full)
        need = workspace_bytes(OP_SOMM, m, k, ld, bs)
        ws = self.workspace(need)
        self._sync_stream()
        flags = (FULL_B if b_full else 0) | (WEIGHTS_NEURON_MAJOR if neuron_major else 0) | planes
        self._check(self.lib.comet_somm_share(self.h, party, m, k, n_full, bs, _ptr(blk_idx),
                                              _ptr(n_blk_dev), n_blk_cap, flags,
                                              _ptr(e), _ptr(f), _ptr(a_i), _ptr(b_i), _ptr(c_i),
                                              _ptr(out), _ptr(ws), need))
        return out

    @staticmethod
    def _somm_shapes(m, k, ld, n_full, f, a_i, b_i, c_i, out, b_full, neuron_major):
        tr = (lambda r, c: (c, r)) if neuron_major else (lambda r, c: (r, c))
        _shape(f, tr(k, ld), "F"), _shape(a_i, (m, k), "A_i")
        _shape(b_i, tr(k, n_full if b_full else ld), "B_i")
        _shape(c_i, (m, ld), "C_i"), _shape(out, (m, ld), "out")

    @staticmethod
    def _simm_shapes(m, n, ld, k_full, e, f, a_i, b_i, c_i, out, a_full, b_full):
        _shape(e, (m, ld), "E"), _shape(f, (ld, n), "F")
        _shape(a_i, (m, k_full if a_full else ld), "A_i")
        _shape(b_i, (k_full if b_full else ld, n), "B_i")
        _shape(c_i, (m, n), "C_i"), _shape(out, (m, n), "out")

    def simm_share(self, party, bs, blk_idx, n_blk_dev, n_blk_cap, e, f, a_i, b_i, c_i,
                   a_full=True, b_full=True, out=None):
        planes = _operands(e, f, a_i, b_i, c_i)
        m = e.shape[0]
        n = f.shape[1]
        ld = n_blk_cap * bs
        k_full = a_i.shape[1] if a_full else (b_i.shape[0] if b_full else 0)
        out = torch.empty((m, n), dtype=torch.int64, device=e.device) if out is None else _words(out, "out")
        self._simm_shapes(m, n, ld, k_full, e, f, a_i, b_i, c_i, out, a_full, b_full)
        _index_list(blk_idx, n_blk_dev, n_blk_cap, a_full or b_full)
        need = workspace_bytes(OP_SIMM, m, ld, n, bs)
        ws = self.workspace(need)
        flags = (FULL_A if a_full else 0) | (FULL_B if b_full else 0) | planes
        self._sync_stream()
        self._check(self.lib.comet_simm_share(self.h, party, m, k_full, n, bs, _ptr(blk_idx),
                                              _ptr(n_blk_dev), n_blk_cap, flags, _ptr(e), _ptr(f),
                                              _ptr(a_i), _ptr(b_i), _ptr(c_i), _ptr(out), _ptr(ws),
                                              need))
        return out

    def somm_share_unopened(self, party, bs, blk_idx, n_blk_dev, n_blk_cap, e, g_0, g_1, a_i, b_i, c_i,
                            b_full=True, out=None):
        """``somm_share`` for at most 8 rows with the opening folded in: ``g_0``, ``g_1`` are the
        two masked shares of the indexed weights (k x ld words), F = g_0 + g_1 is never stored."""
        if _operands(e, g_0, a_i, b_i, c_i) or isinstance(g_1, WeightPlanes):
            raise TypeError("the unopened form takes words, not weight planes")
        m, k = e.shape
        n_full = b_i.shape[1] if b_full else 0
        ld = n_blk_cap * bs
        out = torch.empty((m, ld), dtype=torch.int64, device=e.device) if out is None else _words(out, "out")
        self._somm_shapes(m, k, ld, n_full, g_0, a_i, b_i, c_i, out, b_full, False)
        _shape(_words(g_1, "g_1"), (k, ld), "G_1")
        _index_list(blk_idx, n_blk_dev, n_blk_cap, b_full)
        need = workspace_bytes(OP_SOMM, m, k, ld, bs)
        ws = self.workspace(need)
        self._sync_stream()
        self._check(self.lib.comet_somm_share_unopened(self.h, party, m, k, n_full, bs, _ptr(blk_idx),
                                                       _ptr(n_blk_dev), n_blk_cap, FULL_B if b_full else 0,
                                                       _ptr(e), _ptr(g_0), _ptr(g_1), _ptr(a_i), _ptr(b_i),
                                                       _ptr(c_i), _ptr(out), _ptr(ws), need))
        return out

    def simm_share_unopened(self, party, bs, blk_idx, n_blk_dev, n_blk_cap, e, g_0, g_1, a_i, b_i, c_i,
                            a_full=True, b_full=True, out=None):
        """``simm_share`` for at most 8 rows with the opening folded in (``g_0``, ``g_1``: ld x n)."""
        if _operands(e, g_0, a_i, b_i, c_i) or isinstance(g_1, WeightPlanes):
            raise TypeError("the unopened form takes words, not weight planes")
        m = e.shape[0]
        n = g_0.shape[1]
        ld = n_blk_cap * bs
        k_full = a_i.shape[1] if a_full else (b_i.shape[0] if b_full else 0)
        out = torch.empty((m, n), dtype=torch.int64, device=e.device) if out is None else _words(out, "out")
        self._simm_shapes(m, n, ld, k_full, e, g_0, a_i, b_i, c_i, out, a_full, b_full)
        _shape(_words(g_1, "g_1"), (ld, n), "G_1")
        _index_list(blk_idx, n_blk_dev, n_blk_cap, a_full or b_full)
        need = workspace_bytes(OP_SIMM, m, ld, n, bs)
        ws = self.workspace(need)
        flags = (FULL_A if a_full else 0) | (FULL_B if b_full else 0)
        self._sync_stream()
        self._check(self.lib.comet_simm_share_unopened(self.h, party, m, k_full, n, bs, _ptr(blk_idx),
                                                       _ptr(n_blk_dev), n_blk_cap, flags, _ptr(e), _ptr(g_0),
                                                       _ptr(g_1), _ptr(a_i), _ptr(b_i), _ptr(c_i), _ptr(out),
                                                       _ptr(ws), need))
        return out

    def share_group(self, kind, bs, blk_idx, n_blk_dev, n_blk_cap, members, a_full=True, b_full=True, out=None):
        """Several share products of one shape in one call (``comet_share_group``).  ``kind``:
        "somm" or "simm"; ``members``: a list of ``(party, e, f, a_i, b_i, c_i)``; ``out``: a list
        of output tensors, one per member, or None.  Returns the list of outputs."""
        if kind not in ("somm", "simm"):
            raise ValueError("kind must be 'somm' or 'simm'")
        if not 1 <= len(members) <= SHARE_GROUP_MAX:
            raise ValueError("1 to %d members" % SHARE_GROUP_MAX)
        somm = kind == "somm"
        ld = n_blk_cap * bs
        outs, planes0, dims0 = [], None, None
        arr = (ShareOperands * len(members))()
        for j, (party, e, f, a_i, b_i, c_i) in enumerate(members):
            planes = _operands(e, f, a_i, b_i, c_i)
            if somm:
                m, k = e.shape
                n = b_i.shape[1] if b_full else 0
                zshape = (m, ld)
            else:
                m, n = e.shape[0], f.shape[1]
                k = a_i.shape[1] if a_full else (b_i.shape[0] if b_full else 0)
                zshape = (m, n)
            o = torch.empty(zshape, dtype=torch.int64, device=e.device) if out is None else _words(out[j], "out")
            if somm:
                self._somm_shapes(m, k, ld, n, f, a_i, b_i, c_i, o, b_full, False)
            else:
                self._simm_shapes(m, n, ld, k, e, f, a_i, b_i, c_i, o, a_full, b_full)
            if j == 0:
                planes0, dims0 = planes, (m, k, n)
            elif planes != planes0 or (m, k, n) != dims0:
                raise ValueError("the members of a group have one shape and one operand format")
            arr[j] = ShareOperands(party, 0, *[t.data_ptr() for t in (e, f, a_i, b_i, c_i, o)])
            outs.append(o)
        m, k, n = dims0
        _index_list(blk_idx, n_blk_dev, n_blk_cap, b_full or (a_full and not somm))
        each = workspace_bytes(OP_SOMM, m, k, ld, bs) if somm else workspace_bytes(OP_SIMM, m, ld, n, bs)
        need = each * len(members)
        ws = self.workspace(need)
        flags = planes0 | (FULL_B if b_full else 0) | (FULL_A if (a_full and not somm) else 0)
        self._sync_stream()
        self._check(self.lib.comet_share_group(self.h, OP_SOMM if somm else OP_SIMM, len(members), arr, m, k, n, bs,
                                               _ptr(blk_idx), _ptr(n_blk_dev), n_blk_cap, flags, _ptr(ws), need))
        return outs

    def somm_share_static(self, party, bs, blk_idx, n_blk_dev, n_blk_cap, e, f, a_i, b_i, c_i,
                          b_full=True, neuron_major=False, out=None):
        """``somm_share`` on the library's static scratch array: no workspace, no allocation
        inside the call (pass ``out``, or the result tensor is the one torch allocation)."""
        planes = _operands(e, f, a_i, b_i, c_i)
        m, k = e.shape
        n_full = b_i.shape[0 if neuron_major else 1] if b_full else 0
        ld = n_blk_cap * bs
        out = torch.empty((m, ld), dtype=torch.int64, device=e.device) if out is None else _words(out, "out")
        self._somm_shapes(m, k, ld, n_full, f, a_i, b_i, c_i, out, b_full, neuron_major)
        _index_list(blk_idx, n_blk_dev, n_blk_cap, b_full)
        self._sync_stream()
        flags = (FULL_B if b_full else 0) | (WEIGHTS_NEURON_MAJOR if neuron_major else 0) | planes
        self._check(self.lib.comet_somm_share_static(self.h, party, m, k, n_full, bs, _ptr(blk_idx),
                                                     _ptr(n_blk_dev), n_blk_cap, flags,
                                                     _ptr(e), _ptr(f), _ptr(a_i), _ptr(b_i), _ptr(c_i),
                                                     _ptr(out)))
        return out

    # ---- (4) Protocols 2 and 3 in general form ----
    def components(self, mask):
        """Connected components of the (token, block) graph.  Returns a dict of int32 tensors:
        row_idx, row_comp [n_tok]; blk_idx, blk_comp [nb]; n_row, n_blk, n_comp [1]."""
        if mask.dtype != torch.uint8 or not mask.is_cuda or not mask.is_contiguous() or mask.dim() != 2:
            raise TypeError("mask must be a contiguous 2-D uint8 tensor on the GPU")
        n_tok, nb = mask.shape
        i32 = lambda n: torch.empty(max(n, 1), dtype=torch.int32, device=mask.device)
        out = dict(row_idx=i32(n_tok), row_comp=i32(n_tok), n_row=i32(1), blk_idx=i32(nb),
                   blk_comp=i32(nb), n_blk=i32(1), n_comp=i32(1))
        self._sync_stream()
        self._check(self.lib.comet_components(self.h, _ptr(mask), n_tok, nb, _ptr(out["row_idx"]),
                                              _ptr(out["row_comp"]), _ptr(out["n_row"]),
                                              _ptr(out["blk_idx"]), _ptr(out["blk_comp"]),
                                              _ptr(out["n_blk"]), _ptr(out["n_comp"])))
        return out

    def somm_share_blocks(self, party, bs, blk_idx, blk_comp, n_blk_dev, n_blk_cap, row_comp, n_row_dev,
                          e, f, a_i, b_i, c_i, b_full=True, neuron_major=False, out=None):
        planes = _operands(e, f, a_i, b_i, c_i)
        m, k = e.shape
        n_full = b_i.shape[0 if neuron_major else 1] if b_full else 0
        ld = n_blk_cap * bs
        out = torch.empty((m, ld), dtype=torch.int64, device=e.device) if out is None else _words(out, "out")
        self._somm_shapes(m, k, ld, n_full, f, a_i, b_i, c_i, out, b_full, neuron_major)
        _index_list(blk_idx, n_blk_dev, n_blk_cap, True)
        for t, nm, cnt in ((blk_comp, "blk_comp", 0 if n_blk_dev is not None else n_blk_cap),
                           (row_comp, "row_comp", 0 if n_row_dev is not None else m)):
            if t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous() or t.numel() < cnt:
                raise TypeError("%s must be a contiguous int32 tensor on the GPU with %d entries" % (nm, cnt))
        need = workspace_bytes(OP_SOMM, m, k, ld, bs)
        ws = self.workspace(need)
        self._sync_stream()
        self._check(self.lib.comet_somm_share_blocks(
            self.h, party, m, k, n_full, bs, _ptr(blk_idx), _ptr(blk_comp), _ptr(n_blk_dev), n_blk_cap,
            _ptr(row_comp), _ptr(n_row_dev),
            (FULL_B if b_full else 0) | (WEIGHTS_NEURON_MAJOR if neuron_major else 0) | planes, _ptr(e), _ptr(f), _ptr(a_i),
            _ptr(b_i), _ptr(c_i), _ptr(out), _ptr(ws), need))
        return out

    def simm_share_masked(self, party, bs, blk_idx, n_blk_dev, n_blk_cap, token_mask, e, f, a_i, b_i, c_i,
                          a_full=True, b_full=True, out=None):
        planes = _operands(e, f, a_i, b_i, c_i)
        if token_mask.dtype != torch.uint8 or not token_mask.is_cuda or not token_mask.is_contiguous():
            raise TypeError("token_mask must be a contiguous uint8 tensor on the GPU")
        m = e.shape[0]
        n = f.shape[1]
        if token_mask.dim() != 2 or token_mask.shape[0] != m:
            raise ValueError("token_mask must have one row per row of E")
        ld = n_blk_cap * bs
        k_full = a_i.shape[1] if a_full else (b_i.shape[0] if b_full else 0)
        out = torch.empty((m, n), dtype=torch.int64, device=e.device) if out is None else _words(out, "out")
        self._simm_shapes(m, n, ld, k_full, e, f, a_i, b_i, c_i, out, a_full, b_full)
        _index_list(blk_idx, n_blk_dev, n_blk_cap, True)
        need = workspace_bytes(OP_SIMM, m, ld, n, bs)
        ws = self.workspace(need)
        flags = (FULL_A if a_full else 0) | (FULL_B if b_full else 0) | planes
        self._sync_stream()
        self._check(self.lib.comet_simm_share_masked(
            self.h, party, m, k_full, n, bs, _ptr(blk_idx), _ptr(n_blk_dev), n_blk_cap, flags,
            _ptr(token_mask), token_mask.shape[1], _ptr(e), _ptr(f), _ptr(a_i), _ptr(b_i), _ptr(c_i),
            _ptr(out), _ptr(ws), need))
        return out

    # ---- (5) local steps around the products ----
    def permute_mask(self, src, perm, mask, axis, sign, out=None):
        _words(src, "src"), _words(mask, "mask")
        if perm.dtype != torch.int32 or not perm.is_cuda or not perm.is_contiguous():
            raise TypeError("perm must be a contiguous int32 tensor on the GPU")
        rows, cols = src.shape
        if mask.shape != src.shape or perm.numel() != (cols if axis == AXIS_COLS else rows):
            raise ValueError("mask must have the shape of src and perm one entry per index of the axis")
        out = torch.empty_like(src) if out is None else _words(out, "out")
        self._sync_stream()
        self._check(self.lib.comet_permute_mask(self.h, _ptr(src), _ptr(perm), _ptr(mask), _ptr(out),
                                                rows, cols, axis, sign))
        return out

    def scatter_cols(self, compact, bs, blk_idx, n_blk_dev, n_blk_cap, n_full, out=None):
        _words(compact, "compact")
        m = compact.shape[0]
        if compact.shape[1] != n_blk_cap * bs:
            raise ValueError("compact must be m x n_blk_cap*bs")
        out = torch.empty((m, n_full), dtype=torch.int64, device=compact.device) if out is None \
            else _words(out, "out")
        self._sync_stream()
        self._check(self.lib.comet_scatter_cols(self.h, _ptr(compact), m, bs, _ptr(blk_idx),
                                                _ptr(n_blk_dev), n_blk_cap, _ptr(out), n_full))
        return out

    def truncate_share(self, party, z, frac_bits=16, out=None):
        _words(z, "z")
        out = torch.empty_like(z) if out is None else _words(out, "out")
        self._sync_stream()
        self._check(self.lib.comet_truncate_share(self.h, party, _ptr(z), _ptr(out), z.numel(), frac_bits))
        return out

    # ---- probes ----
    def set_tuning(self, key: int, value: int):
        self._check(self.lib.comet_set_tuning(self.h, key, value))

    def timing_begin(self, max_launches: int):
        self._check(self.lib.comet_timing_begin(self.h, max_launches))

    def timing_end(self):
        ms, n = ctypes.c_double(), ctypes.c_int()
        self._check(self.lib.comet_timing_end(self.h, ctypes.byref(ms), ctypes.byref(n)))
        return ms.value, n.value

    def probe_mfma_i8(self, blocks: int, iters: int, random_operands: bool = False) -> float:
        out = torch.empty(blocks * 256, dtype=torch.int32, device="cuda:%d" % self.device)
        macs = ctypes.c_double()
        self._sync_stream()
        self._check(self.lib.comet_probe_mfma_i8(self.h, blocks, iters, int(random_operands), _ptr(out),
                                                 ctypes.byref(macs)))
        return macs.value

    def probe_valu_mac64(self, blocks: int, iters: int) -> float:
        out = torch.empty(blocks * 256, dtype=torch.int64, device="cuda:%d" % self.device)
        macs = ctypes.c_double()
        self._sync_stream()
        self._check(self.lib.comet_probe_valu_mac64(self.h, blocks, iters, _ptr(out), ctypes.byref(macs)))
        return macs.value

    def probe_copy(self, src, dst):
        self._sync_stream()
        self._check(self.lib.comet_probe_copy(self.h, _ptr(src), _ptr(dst), src.numel()))
        return dst
