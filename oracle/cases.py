"""Assemble complete two-party test cases from the raw synthetic draws.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  The data owner's role
(fixed-point encoding, share splitting) and the trusted third party's role
(triples) are played here with oracle arithmetic; the raw random draws come
from ``workloads``.
"""
from __future__ import annotations

import numpy as np

import oracle as co
from oracle import protocols
from workloads import configs, rng

FRAC_BITS = 16


def build(cfg: configs.Config, mm: configs.MatMul, seed: int = rng.BASE_SEED,
          with_result: bool = True, mask: np.ndarray | None = None):
    """Return ``(case, plain)``: the :class:`protocols.BlockCase` for matmul
    ``mm`` of ``cfg`` and a dict with the plaintext float and encoded secrets."""
    raw = configs.raw_inputs(cfg, mm, seed)
    xq = co.encode(raw["x"], FRAC_BITS)
    yq = co.encode(raw["y"], FRAC_BITS)
    x_sh = co.share(xq, raw["x_split"])
    y_sh = co.share(yq, raw["y_split"])
    if mask is None:
        mask = configs.token_masks(cfg, seed)
    n_kept = int(np.count_nonzero(mask.max(axis=0))) * cfg.bs
    rows, cols = (mm.m, n_kept) if mm.kind == "somm" else (mm.m, mm.n)
    c_split = configs.c_split(cfg, mm, rows, cols, seed)
    case = protocols.block_case(mm.kind, x_sh, y_sh, mask, cfg.bs, raw["a"], raw["b"],
                                raw["a_split"], raw["b_split"], c_split, with_result)
    plain = dict(x=raw["x"], y=raw["y"], xq=xq, yq=yq, mask=mask)
    return case, plain
