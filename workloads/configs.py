"""The five synthetic FFN workloads and their raw random inputs.

Shapes follow public model dimensions (OPT-125m, LLaMA-7B, LLaMA-2-13B); the
paper's own workloads (Sec. 7.1: prompts run through trained OPT / Llama2
checkpoints) are not available offline, so seeded synthetic data of the same
shape and statistics stands in for them.

A matmul is described in the notation of the paper's Sec. 5: ``Z = X Y`` with
``X`` of shape ``m x k`` (activations) and ``Y`` of shape ``k x n`` (weights).
``kind == "somm"`` restricts the *output* columns (Protocol 2: FC1 / gate /
up), ``kind == "simm"`` restricts the *contraction* axis (Protocol 3: FC2 /
down).  This module returns raw random draws only; fixed-point encoding, share
splitting and triple generation are done by whoever consumes them.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List

import numpy as np

from . import masks, rng

# stream roles
R_X, R_Y, R_XSPLIT, R_YSPLIT, R_A, R_B, R_ASPLIT, R_BSPLIT, R_CSPLIT, R_MASK = range(10)
R_TOKEN_MASK = 100


@dataclass(frozen=True)
class MatMul:
    name: str
    kind: str          # "somm" | "simm"
    m: int
    k: int             # full contraction length
    n: int             # full output width
    index: int         # matrix index inside the config (seeds)


@dataclass(frozen=True)
class Config:
    cid: int
    name: str
    d_model: int
    d_ff: int
    tokens: int
    bs: int
    density: float
    mask_kind: str     # "uniform" | "clustered" | "per_token_union"
    matmuls: List[MatMul] = field(default_factory=list)

    @property
    def nb(self) -> int:
        return self.d_ff // self.bs


def _ffn(cid, name, d, f, m, bs, density, mask_kind, names):
    mm = []
    for i, nm in enumerate(names):
        if nm == "down":
            mm.append(MatMul(nm, "simm", m, f, d, i))
        else:
            mm.append(MatMul(nm, "somm", m, d, f, i))
    return Config(cid, name, d, f, m, bs, density, mask_kind, mm)


def config(cid: int, density: float | None = None) -> Config:
    """Config ``cid`` in 1..5.  ``density`` overrides the default (config 5 sweep)."""
    if cid == 1:
        return _ffn(1, "tiny", 64, 256, 16, 16, 0.25, "uniform", ["up", "down"])
    if cid == 2:
        return _ffn(2, "opt125m", 768, 3072, 128, 32, 0.10, "clustered", ["up", "down"])
    if cid == 3:
        return _ffn(3, "llama7b", 4096, 11008, 256, 32, 0.15, "clustered", ["gate", "up", "down"])
    if cid == 4:
        return _ffn(4, "llama13b_decode", 5120, 13824, 8, 64, 0.20, "per_token_union",
                    ["gate", "up", "down"])
    if cid == 5:
        d = 1.0 if density is None else density
        return _ffn(5, "llama7b_down_d%03d" % round(d * 100), 4096, 11008, 512, 32, d,
                    "clustered", ["down"])
    raise ValueError("config id must be 1..5")


C5_DENSITIES = (1.0, 0.5, 0.25, 0.10, 0.05)


def stream_id(cfg: Config, matrix: int, role: int) -> int:
    # config 5's density variants share streams on purpose: same matrices, different mask
    return 100000 * cfg.cid + 1000 * matrix + role


def token_masks(cfg: Config, seed: int = rng.BASE_SEED) -> np.ndarray:
    """Per-token block masks ``[n_tok, nb]`` (uint8).  One row unless the
    config draws an independent mask per token (decode batch)."""
    sid = stream_id(cfg, 0, R_MASK)
    if cfg.mask_kind == "uniform":
        return masks.uniform_block_mask(seed, sid, cfg.nb, cfg.density)[None, :]
    if cfg.mask_kind == "clustered":
        return masks.clustered_block_mask(seed, sid, cfg.nb, cfg.density)[None, :]
    if cfg.mask_kind == "per_token_union":
        return masks.per_token_masks(seed, stream_id(cfg, 0, R_TOKEN_MASK), cfg.tokens,
                                     cfg.nb, cfg.density, clustered=False)
    raise ValueError(cfg.mask_kind)


def raw_inputs(cfg: Config, mm: MatMul, seed: int = rng.BASE_SEED,
               secrets: bool = True) -> Dict[str, np.ndarray]:
    """Raw draws for one matmul.

    ``x``, ``y``: float64 N(0,1) secrets (omitted when ``secrets`` is False);
    ``x_split``, ``y_split``, ``a``, ``b``, ``a_split``, ``b_split``: uniform
    uint64 at full shape (share-splitting randomness and triple parts);
    ``c_split`` is drawn lazily by :func:`c_split` once the compact output
    shape is known.
    """
    out: Dict[str, np.ndarray] = {}
    mk, kn = mm.m * mm.k, mm.k * mm.n
    sid = lambda role: stream_id(cfg, mm.index, role)
    if secrets:
        out["x"] = rng.gaussian_f64(seed, sid(R_X), mk).reshape(mm.m, mm.k)
        out["y"] = rng.gaussian_f64(seed, sid(R_Y), kn).reshape(mm.k, mm.n)
    out["x_split"] = rng.uniform_u64(seed, sid(R_XSPLIT), mk).reshape(mm.m, mm.k)
    out["y_split"] = rng.uniform_u64(seed, sid(R_YSPLIT), kn).reshape(mm.k, mm.n)
    out["a"] = rng.uniform_u64(seed, sid(R_A), mk).reshape(mm.m, mm.k)
    out["b"] = rng.uniform_u64(seed, sid(R_B), kn).reshape(mm.k, mm.n)
    out["a_split"] = rng.uniform_u64(seed, sid(R_ASPLIT), mk).reshape(mm.m, mm.k)
    out["b_split"] = rng.uniform_u64(seed, sid(R_BSPLIT), kn).reshape(mm.k, mm.n)
    return out


def c_split(cfg: Config, mm: MatMul, rows: int, cols: int, seed: int = rng.BASE_SEED) -> np.ndarray:
    """Uniform uint64 randomness that splits the triple's C into two shares."""
    return rng.uniform_u64(seed, stream_id(cfg, mm.index, R_CSPLIT), rows * cols).reshape(rows, cols)


# ---------------------------------------------------------------------------
# MHA-shaped workload (Sec. 3.1 workflow, Sec. 6): head-granular sparsity
# ---------------------------------------------------------------------------

@dataclass(frozen=True)
class MhaConfig:
    """Sparse QKV layer (Protocol 2) and sparse output layer (Protocol 3) of one attention
    module with head-granular sparsity: a block is one attention head (``bs = head_dim``).

    Rows of the QKV product are the tokens of the current step plus the merged cache-refill
    requests of Sec. 6.1 (one row per token whose keys / values are missing for some heads), so
    every row carries its own set of heads.  The fused QKV weight has ``3 * n_heads`` column
    blocks (Q heads, then K heads, then V heads); a head that is active for a row keeps its
    three blocks."""
    name: str
    d_model: int
    n_heads: int
    head_dim: int
    tokens: int          # tokens of the current step (every activated head: Q, K and V)
    refill_rows: int     # merged cache-miss rows (K and V of the heads they miss)
    head_density: float  # fraction of heads a token activates ("more than 50 % inactive", Sec. 2.3)

    @property
    def rows(self) -> int:
        return self.tokens + self.refill_rows


def mha_config() -> MhaConfig:
    """LLaMA-2-7B attention shape: 32 heads of 128, decode batch of 8 with 56 refill rows."""
    return MhaConfig("llama7b_mha", 4096, 32, 128, 8, 56, 0.5)


def mha_head_masks(cfg: MhaConfig, seed: int = rng.BASE_SEED):
    """(qkv_mask [rows, 3 * n_heads], out_mask [tokens, n_heads]) as uint8.

    Current tokens activate ``head_density`` of the heads, chosen uniformly per token (heads show
    no spatial locality); a refill row misses between one and four of the heads that the current
    step uses, and asks for their K and V blocks only."""
    h = cfg.n_heads
    out_mask = np.stack([masks.uniform_block_mask(seed, 6000 + t, h, cfg.head_density)
                         for t in range(cfg.tokens)])
    used = np.nonzero(out_mask.max(axis=0))[0]
    qkv = np.zeros((cfg.rows, 3 * h), dtype=np.uint8)
    qkv[:cfg.tokens, 0:h] = out_mask
    qkv[:cfg.tokens, h:2 * h] = out_mask
    qkv[:cfg.tokens, 2 * h:3 * h] = out_mask
    draws = rng.uniform_u64(seed, 6500, cfg.refill_rows * 5).reshape(cfg.refill_rows, 5)
    for r in range(cfg.refill_rows):
        n_miss = 1 + int(draws[r, 0] % np.uint64(4))
        for j in range(n_miss):
            head = int(used[int(draws[r, 1 + j] % np.uint64(len(used)))])
            qkv[cfg.tokens + r, h + head] = 1          # K of that head
            qkv[cfg.tokens + r, 2 * h + head] = 1      # V of that head
    return qkv, out_mask
