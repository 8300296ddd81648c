"""Decision margins for parity inputs.  TEST INFRASTRUCTURE ONLY (sits with the oracle).

Bit-exact comparison of integer outputs (keep mask, arg max, anchor index) between a
float32 GPU path and the float64 oracle only means something when no decision sits on a
rounding knife-edge.  This helper judges a generated batch with the oracle and asks the
generator to redraw every source token whose best similarity is within ``sim_margin`` of a
threshold, or whose best and second-best candidates are closer than ``top2_margin``; it
then checks that the anchor rule's best two frame scores differ by at least ``anchor_gap``.
Source tokens never influence each other's matches, so redrawing converges in a few rounds.
"""
from __future__ import annotations

from typing import Sequence

import numpy as np

from . import ttf_oracle as orc


class MarginError(RuntimeError):
    pass


def violators(res: "orc.OracleResult", ts: Sequence[float], sim_margin: float,
              top2_margin: float) -> np.ndarray:
    """[n,3] array of (b,k,i) of source tokens that break a margin."""
    B, F, N = res.best_sim.shape
    src = np.ones((B, F, N), bool)
    for b in range(B):
        src[b, res.anchor_index[b]] = False
    bad = np.zeros((B, F, N), bool)
    for t in ts:
        bad |= np.abs(res.best_sim - float(np.float32(t))) < sim_margin
    bad |= (res.best_sim - res.second_sim) < top2_margin
    bad &= src
    return np.argwhere(bad).astype(np.int32)


def anchor_gap(res: "orc.OracleResult") -> float:
    """Smallest (best - runner-up) frame score over the clips (inf when F == 1)."""
    B, F = res.anchor_score.shape
    if F < 2:
        return float("inf")
    s = np.sort(res.anchor_score, axis=1)
    return float((s[:, -1] - s[:, -2]).min())


def enforce_margins(batch, r: int, ts: Sequence[float], anchor_mode: int = orc.ANCHOR_AUTO,
                    anchor_index: int = 0, sim_margin: float = 1e-3, top2_margin: float = 1e-4,
                    gap: float = 1e-4, max_rounds: int = 8, want_tokens: bool = True):
    """Redraw margin-breaking tokens of ``batch`` in place; return the final OracleResult
    for ts[0].  Raises MarginError if a margin cannot be met (caller picks another seed)."""
    res = orc.compress(batch.x, r, ts[0], anchor_mode, anchor_index, want_tokens=False)
    todo = violators(res, ts, sim_margin, top2_margin)
    rounds = 0
    while len(todo):
        if rounds >= max_rounds:
            raise MarginError(f"{len(todo)} tokens still inside the margins after {rounds} rounds")
        batch.redraw([tuple(int(v) for v in row) for row in todo], batch.redraw_rounds)
        rounds += 1
        best, second, _ = orc.match_tokens(batch.x, r, res.anchor_index, todo)
        bad = np.zeros(len(todo), bool)
        for t in ts:
            bad |= np.abs(best - float(np.float32(t))) < sim_margin
        bad |= (best - second) < top2_margin
        todo = todo[bad]
    final = orc.compress(batch.x, r, ts[0], anchor_mode, anchor_index, want_tokens=want_tokens)
    left = violators(final, ts, sim_margin, top2_margin)
    if len(left):
        raise MarginError(f"{len(left)} tokens inside the margins after the final pass")
    if anchor_mode == orc.ANCHOR_AUTO and anchor_gap(final) < gap:
        raise MarginError(f"anchor score gap {anchor_gap(final):.3g} below {gap:g}")
    return final


def enforce_tied_margins(batch, r: int, ts: Sequence[float], anchor_mode: int = orc.ANCHOR_AUTO,
                         anchor_index: int = 0, sim_margin: float = 1e-3, top2_margin: float = 1e-4,
                         gap: float = 1e-4, max_rounds: int = 8, want_tokens: bool = True):
    """Tied-batch counterpart of enforce_margins: a source position is redrawn (in every batch
    element) while its two best batch-mean similarities are closer than ``top2_margin`` or any
    element's similarity at the shared offset is within ``sim_margin`` of a threshold.  Returns
    the final TiedResult for ts[0]."""
    B = batch.x.shape[0]
    for rounds in range(max_rounds + 1):
        res = orc.compress_tied(batch.x, r, ts[0], anchor_mode, anchor_index, want_tokens=False)
        F, N = res.fuse_map.shape
        bad = (res.mean_sim - res.second_mean) < top2_margin
        for t in ts:
            bad |= (np.abs(res.best_sim - float(np.float32(t))) < sim_margin).any(axis=0)
        bad[res.anchor_index] = False
        todo = np.argwhere(bad)
        if len(todo) == 0:
            break
        if rounds == max_rounds:
            raise MarginError(f"{len(todo)} positions still inside the margins after {rounds} rounds")
        batch.redraw([(b, int(k), int(i)) for (k, i) in todo for b in range(B)], batch.redraw_rounds)
    if anchor_mode == orc.ANCHOR_AUTO and F > 1:
        s = np.sort(res.anchor_score)
        if s[-1] - s[-2] < gap:
            raise MarginError(f"anchor score gap {s[-1] - s[-2]:.3g} below {gap:g}")
    return orc.compress_tied(batch.x, r, ts[0], anchor_mode, anchor_index, want_tokens=want_tokens)
