"""Oracle for video-adaptive threshold selection.  TEST INFRASTRUCTURE ONLY.

Discussion D1 proposes to calibrate the threshold t per clip from the empirical distribution
of the best-match similarities {s^(k,i)} and leaves the rule open.  The rule implemented here
is an order statistic: for a requested fused fraction phi in [0,1] of the M = (F-1) N source
tokens of a clip,

    rank = clamp(ceil((1 - phi) * M), 1, M),      t = the rank-th smallest s^ of the clip,

so that a token is fused (s^ > t) only if it lies strictly above that order statistic; at most
floor(phi * M) tokens are fused, exactly that many when the values around the rank are
distinct.  A clip without source tokens (F = 1) gets t = 1.  Similarities are ordered as the
real numbers they are; inputs are assumed free of NaN.
"""
from __future__ import annotations

import math

import numpy as np


def rank_for_fraction(fraction: float, M: int) -> int:
    """1-based rank of the order statistic; the product is formed in double precision from
    the float32 value of `fraction`."""
    phi = float(np.float32(fraction))
    return max(1, min(M, int(math.ceil((1.0 - phi) * M))))


def select_threshold(best_sim: np.ndarray, anchor_index: np.ndarray, fraction: float) -> np.ndarray:
    """best_sim [B,F,N] (any float type) -> t [B] in the same type."""
    B, F, N = best_sim.shape
    t = np.ones(B, best_sim.dtype)
    for b in range(B):
        a = int(anchor_index[b])
        src = np.concatenate([best_sim[b, k] for k in range(F) if k != a]) if F > 1 else np.zeros(0)
        M = src.size
        if M == 0:
            continue
        t[b] = np.sort(src)[rank_for_fraction(fraction, M) - 1]
    return t


def compress_per_clip(x: np.ndarray, r: int, thresholds, anchor_index):
    """The whole pass with clip b gated at thresholds[b] and its anchor fixed to
    anchor_index[b]: every clip is an independent B=1 problem, so this is one plain run per
    clip, packed clip after clip like the batched pass."""
    from . import ttf_oracle as T
    B, F, H, W, C = x.shape
    N, cap = H * W, B * F * H * W
    parts = [T.compress(x[b:b + 1], r, float(thresholds[b]), T.ANCHOR_FIXED, int(anchor_index[b]))
             for b in range(B)]
    rows = [p.total_rows for p in parts]
    off = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    src = np.full(cap, -1, np.int32)
    pos = np.full((3, cap), -1, np.int32)
    tok = np.zeros((cap, C), x.dtype)
    for b, p in enumerate(parts):
        src[off[b]:off[b + 1]] = p.src_index[:rows[b]]
        pos[:, off[b]:off[b + 1]] = p.pos_ids[:, :rows[b]]
        tok[off[b]:off[b + 1]] = p.tokens_out[:rows[b]]
    cat = lambda name: np.concatenate([getattr(p, name) for p in parts], axis=0)
    return T.OracleResult(
        anchor_index=cat("anchor_index"), anchor_score=cat("anchor_score"), best_sim=cat("best_sim"),
        second_sim=cat("second_sim"), best_idx=cat("best_idx"), cand_count=cat("cand_count"),
        fuse_map=cat("fuse_map"), kept_count=np.asarray(rows, np.int32), row_offsets=off,
        src_index=src, pos_ids=pos, tokens_out=tok)
