"""Oracle for segment-wise (streaming) compression.  TEST INFRASTRUCTURE ONLY.

The streaming use of Discussion D3: a video is handled piece by piece, and a piece is matched
against the frame that closed the piece before it instead of a frame of its own, so that nothing
already emitted is touched again.  A segment of F frames with an external anchor frame is therefore the
plain pass on the (F+1)-frame clip [anchor ; segment] with the anchor fixed to its first
frame, minus the N anchor rows (they were emitted when that frame was a source frame of the
previous segment): every segment frame is a source frame, the output holds only the preserved
source rows in ascending flat order, and the temporal coordinate of frame k of the segment is
frame_offset + k.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class SegmentResult:
    best_sim: np.ndarray      # [B,F,N] float64
    second_sim: np.ndarray    # [B,F,N] float64
    best_idx: np.ndarray      # [B,F,N] int32, flat index in the external anchor frame
    fuse_map: np.ndarray      # [B,F,N] int32
    kept_count: np.ndarray    # [B]     int32, P of every clip
    row_offsets: np.ndarray   # [B+1]   int32
    src_index: np.ndarray     # [B*F*N] int32, k*N+i inside the segment
    pos_ids: np.ndarray       # [3,B*F*N] int32, temporal plane = frame_offset + k
    tokens_out: np.ndarray    # [B*F*N, C]

    @property
    def total_rows(self) -> int:
        return int(self.row_offsets[-1])


def compress_segment(x: np.ndarray, anchor_frame: np.ndarray, r: int, t: float,
                     frame_offset: int = 0) -> SegmentResult:
    """x [B,F,H,W,C], anchor_frame [B,H,W,C] of the same element type."""
    from . import ttf_oracle as T
    B, F, H, W, C = x.shape
    N, cap = H * W, B * F * H * W
    clip = np.concatenate([anchor_frame[:, None], x], axis=1)
    res = T.compress(clip, r, t, T.ANCHOR_FIXED, 0)
    src = np.full(cap, -1, np.int32)
    pos = np.full((3, cap), -1, np.int32)
    tok = np.zeros((cap, C), x.dtype)
    off = np.zeros(B + 1, np.int32)
    for b in range(B):
        first, last = int(res.row_offsets[b]) + N, int(res.row_offsets[b + 1])   # skip the anchor rows
        n = last - first
        o = int(off[b])
        src[o:o + n] = res.src_index[first:last] - N
        pos[:, o:o + n] = res.pos_ids[:, first:last]
        pos[0, o:o + n] += frame_offset - 1
        tok[o:o + n] = res.tokens_out[first:last]
        off[b + 1] = o + n
    return SegmentResult(best_sim=res.best_sim[:, 1:], second_sim=res.second_sim[:, 1:],
                         best_idx=res.best_idx[:, 1:], fuse_map=res.fuse_map[:, 1:],
                         kept_count=np.diff(off).astype(np.int32), row_offsets=off,
                         src_index=src, pos_ids=pos, tokens_out=tok)
