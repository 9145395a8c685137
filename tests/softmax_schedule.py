"""Host model of when a tiled online softmax has to move its reference point (test helper).

The fused attention forward walks the keys in tiles of 64 and keeps, per query, a reference
exponent in log2 units.  A wave of 32 consecutive queries moves its references (and rescales the
running sums and output accumulators) at a key tile only when some query of the wave has a score in
that tile more than 2^8 above its reference; otherwise the old reference stays.  The first tile
always sets the reference, so the interesting events are the moves at LATER tiles: inputs that never
cause one do not test the rescaling at all.

`rescale_stats` replays that rule on the oracle's logits (fp64, natural-log units) and reports how
often it fires, so that a stress test can assert that it really is a stress.  It knows the tile
shapes (32 queries per wave, 64 keys per tile, threshold 8) and nothing else of the kernel.
"""
from __future__ import annotations

import numpy as np

LOG2E = 1.4426950408889634
QUERIES_PER_WAVE, KEYS_PER_TILE, THRESHOLD_LOG2 = 32, 64, 8.0


def rescale_stats(logits: np.ndarray) -> dict:
    """logits [..., Nq, Nk] in natural-log units, -inf where masked.  Returns counts over all
    (wave, key tile) steps: `steps_late` = steps at key tiles after the first that hold at least one
    unmasked key for the wave, `moves_late` = those at which the reference moves, `max_rise_log2` = the
    largest rise of a reference at a late move, `mean_max_prob` = mean over queries of the largest
    softmax probability."""
    s = np.asarray(logits, dtype=np.float64) * LOG2E
    s = s.reshape((-1,) + s.shape[-2:])
    n_bh, nq, nk = s.shape
    moves = steps = 0
    max_rise = 0.0
    for bh in range(n_bh):
        for q0 in range(0, nq, QUERIES_PER_WAVE):
            blk = s[bh, q0:q0 + QUERIES_PER_WAVE]
            ref = np.full(blk.shape[0], -np.inf)
            for t, k0 in enumerate(range(0, nk, KEYS_PER_TILE)):
                tile_max = blk[:, k0:k0 + KEYS_PER_TILE].max(axis=1)
                if not np.isfinite(tile_max).any():
                    continue                      # a causal wave never reaches this tile
                cand = np.maximum(ref, tile_max)
                with np.errstate(invalid="ignore"):
                    bump = bool(np.any(cand > ref + THRESHOLD_LOG2))
                if t > 0:
                    steps += 1
                    if bump:
                        moves += 1
                        rise = cand - ref
                        rise = rise[np.isfinite(rise)]
                        if rise.size:
                            max_rise = max(max_rise, float(rise.max()))
                if bump:
                    ref = cand
    m = s.max(axis=-1, keepdims=True)
    p = np.exp2(s - m)
    p /= p.sum(axis=-1, keepdims=True)
    return {"steps_late": steps, "moves_late": moves, "max_rise_log2": max_rise,
            "mean_max_prob": float(p.max(axis=-1).mean())}


def head_logits(q: np.ndarray, k: np.ndarray, n_heads: int, causal: bool = False) -> np.ndarray:
    """q [B, Nq, d], k [B, Nk, d] -> logits [B, H, Nq, Nk] = q k^T / sqrt(d_head), -inf above the
    diagonal when causal (the definition the oracle's attention uses)."""
    B, Nq, d = q.shape
    Nk, dh = k.shape[1], d // n_heads
    qh = q.reshape(B, Nq, n_heads, dh)
    kh = k.reshape(B, Nk, n_heads, dh)
    s = np.einsum("bqhd,bkhd->bhqk", qh, kh) / np.sqrt(dh)
    if causal:
        s = np.where(np.arange(Nk)[None, :] > np.arange(Nq)[:, None], -np.inf, s)
    return s
