"""Seeded synthetic block masks standing in for the predictor's output.

The paper's predictor (Sec. 4.1) needs trained weights and real prompts, so
its output -- a plaintext 0/1 sparsity distribution in an arbitrary fixed
order (Sec. 4.2, Sec. 5 opening) -- is replaced by a seeded mask over blocks
of ``bs`` consecutive FFN neurons.  Masks are ``uint8`` arrays of 0/1 flags.
No protocol arithmetic lives here.
"""
from __future__ import annotations

import math

import numpy as np

from . import rng


def kept_blocks(density: float, nb: int) -> int:
    """Exact number of active blocks for a target density (round half up)."""
    return min(nb, int(math.floor(density * nb + 0.5)))


def uniform_block_mask(seed: int, stream_id: int, nb: int, density: float) -> np.ndarray:
    """Exactly ``kept_blocks`` active blocks, chosen uniformly at random."""
    t = kept_blocks(density, nb)
    keys = rng.uniform_u64(seed, stream_id, nb)
    order = np.argsort(keys, kind="stable")
    mask = np.zeros(nb, dtype=np.uint8)
    mask[order[:t]] = 1
    return mask


def clustered_block_mask(seed: int, stream_id: int, nb: int, density: float,
                         mean_run: float = 4.0) -> np.ndarray:
    """Exactly ``kept_blocks`` active blocks laid down as contiguous runs.

    Repeats: start ~ U[0, nb), run length L ~ Geometric(p = 1/mean_run) on
    {1, 2, ...}; blocks ``start .. min(start+L, nb)`` that are still inactive
    are activated one by one, stopping the moment the count reaches the
    target.  No wrap-around.  Models the spatial locality of activation
    sparsity that Sec. 5 of the paper relies on.
    """
    t = kept_blocks(density, nb)
    mask = np.zeros(nb, dtype=np.uint8)
    if t >= nb:
        mask[:] = 1
        return mask
    p = 1.0 / mean_run
    log1mp = math.log1p(-p)
    count = 0
    drawn = 0
    batch = 256
    while count < t:
        u = rng.uniform_01(seed, stream_id, 2 * batch, offset=drawn)
        drawn += 2 * batch
        for i in range(batch):
            start = min(nb - 1, int(u[2 * i] * nb))
            run = 1 + int(math.floor(math.log(u[2 * i + 1]) / log1mp))
            for b in range(start, min(start + run, nb)):
                if not mask[b]:
                    mask[b] = 1
                    count += 1
                    if count == t:
                        return mask
    return mask


def per_token_masks(seed: int, stream_base: int, n_tok: int, nb: int, density: float,
                    clustered: bool = True) -> np.ndarray:
    """Independent masks for ``n_tok`` tokens, shape ``[n_tok, nb]``."""
    gen = clustered_block_mask if clustered else uniform_block_mask
    return np.stack([gen(seed, stream_base + t, nb, density) for t in range(n_tok)])


def stress_mask(seed: int, stream_id: int, n_flags: int, density: float = 0.15,
                mean_run: float = 4.0) -> np.ndarray:
    """Large clustered mask for bandwidth measurements (vectorised recipe).

    Run starts are Bernoulli with rate ``density / mean_run`` per position and
    run lengths Geometric(1/mean_run); overlapping runs merge, so the realised
    density is a little below the target.  Only the statistics matter here.
    """
    p_start = density / mean_run
    out = np.zeros(n_flags + 1, dtype=np.int32)
    chunk = 1 << 24
    log1mp = math.log1p(-1.0 / mean_run)
    for s in range(0, n_flags, chunk):
        e = min(n_flags, s + chunk)
        u = rng.uniform_01(seed, stream_id, e - s, offset=s)
        starts = np.nonzero(u < p_start)[0]
        v = rng.uniform_01(seed, stream_id + 1, e - s, offset=s)[starts]
        runs = 1 + np.floor(np.log(v) / log1mp).astype(np.int64)
        ends = np.minimum(starts + s + runs, n_flags)
        np.add.at(out, starts + s, 1)
        np.add.at(out, ends, -1)
    return (np.cumsum(out[:n_flags]) > 0).astype(np.uint8)


def stress_mask_device(seed: int, n_flags: int, device, density: float = 0.15,
                       mean_run: float = 4.0):
    """The recipe of :func:`stress_mask`, drawn with torch's seeded generator on
    ``device`` (host generation of 2^28 flags would take most of a minute).
    Returns a uint8 tensor of 0/1 flags."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    p_start = density / mean_run
    starts = (torch.rand(n_flags, device=device, generator=gen) < p_start).nonzero().squeeze(1)
    v = torch.rand(starts.numel(), device=device, generator=gen).clamp_(min=1e-12)
    runs = 1 + torch.floor(torch.log(v) / math.log1p(-1.0 / mean_run)).to(torch.int64)
    ends = torch.clamp(starts + runs, max=n_flags)
    delta = torch.zeros(n_flags + 1, dtype=torch.int32, device=device)
    one = torch.ones(starts.numel(), dtype=torch.int32, device=device)
    delta.index_add_(0, starts, one)
    delta.index_add_(0, ends, -one)
    return (torch.cumsum(delta[:n_flags], 0, dtype=torch.int32) > 0).to(torch.uint8)


def grouped_token_masks(seed: int, stream_base: int, n_tok: int, nb: int, groups: int,
                        density: float, mean_run: float = 4.0) -> np.ndarray:
    """Per-token masks whose (token, block) graph has several connected components.

    Token ``t`` belongs to group ``t * groups // n_tok`` (think of a batch that holds ``groups``
    unrelated requests); a group owns the block range ``[g * nb // groups, (g + 1) * nb // groups)``
    and each of its tokens draws an independent clustered mask inside that range with
    ``density * groups`` of the range active, i.e. ``density`` of all blocks.  Tokens of a group
    overlap, tokens of different groups never do: the setting in which Protocol 2's grouping
    into result blocks saves computation over the union of all masks.  Shape ``[n_tok, nb]``."""
    out = np.zeros((n_tok, nb), dtype=np.uint8)
    for t in range(n_tok):
        g = t * groups // n_tok
        lo, hi = g * nb // groups, (g + 1) * nb // groups
        d = min(1.0, density * groups)
        out[t, lo:hi] = clustered_block_mask(seed, stream_base + t, hi - lo, d, mean_run)
    return out
