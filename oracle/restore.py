"""Oracle for token restoration and decode alignment.  TEST INFRASTRUCTURE ONLY.

Restoration (Discussion D4, "TTF-R"): the compressed sequence is expanded back to the full
[F, N] layout through the mapping dst(k,i) of the matching step: a retained token is its own
row, a fused token is represented by the anchor token it was matched to.  Since the stacked X'
puts the N anchor rows first, in grid order, the anchor token with flat index j is row j of
its clip.

Decode alignment (Section 3, "Cache-aware Decode Alignment"): L_pre = L' + T, the position of
decode step l is L_pre + l and the attention mask then spans L_pre + l + 1 entries.
"""
from __future__ import annotations

import numpy as np


def restore_map(fuse_map: np.ndarray, anchor_index: np.ndarray, row_offsets: np.ndarray,
                src_index: np.ndarray) -> np.ndarray:
    """[B,F,N] int32: the output row that stands for every original token."""
    B, F, N = fuse_map.shape
    out = np.full((B, F, N), -1, np.int32)
    for b in range(B):
        first, last = int(row_offsets[b]), int(row_offsets[b + 1])
        flat = out[b].reshape(-1)
        for row in range(first, last):                 # retained tokens: their own row
            flat[int(src_index[row])] = row
        a = int(anchor_index[b])
        for k in range(F):
            if k == a:
                continue
            for i in range(N):
                j = int(fuse_map[b, k, i])
                if j >= 0:                             # fused: the anchor row of dst(k,i)
                    out[b, k, i] = first + j
    return out


def restore(tokens_out: np.ndarray, rmap: np.ndarray) -> np.ndarray:
    """[B,F,N,C]: every original position filled with the row that represents it."""
    return tokens_out[rmap]


def decode_alignment(l_prime: int, text_tokens: int, step: int):
    """(L_pre, position of decode step `step`, attention-mask length at that step)."""
    l_pre = int(l_prime) + int(text_tokens)
    return l_pre, l_pre + int(step), l_pre + int(step) + 1
