"""Second, independently written evaluation of the TTF definition in NumPy float64.

Formulated differently from the C oracle on purpose: the full N x N cosine matrix of a source
frame against the anchor frame (normalised matrix product, i.e. the "global matching" the
paper contrasts with in its introduction), then restricted to pairs whose grid distance is at
most r in both axes.  Used only to pin the oracle on small inputs.
"""
import numpy as np


def cos_matrix(u: np.ndarray, v: np.ndarray) -> np.ndarray:
    """All-pairs cosine between rows of u [n,C] and rows of v [m,C]; 0 where a norm is 0."""
    nu = np.linalg.norm(u, axis=1)
    nv = np.linalg.norm(v, axis=1)
    den = nu[:, None] * nv[None, :]
    dots = u @ v.T
    return np.divide(dots, den, out=np.zeros_like(dots), where=den > 0)


def window_mask(H: int, W: int, r: int) -> np.ndarray:
    """[N,N] True where anchor token j lies within the (2r+1)^2 window centred on token i."""
    ys, xs = np.divmod(np.arange(H * W), W)
    return (np.abs(ys[:, None] - ys[None, :]) <= r) & (np.abs(xs[:, None] - xs[None, :]) <= r)


def anchor_scores(clip: np.ndarray) -> np.ndarray:
    """clip [F,N,C] float64 -> cosine of each frame's mean token with the clip's mean token."""
    frame_mean = clip.mean(axis=1)
    clip_mean = clip.reshape(-1, clip.shape[-1]).mean(axis=0)
    return cos_matrix(frame_mean, clip_mean[None])[:, 0]


def ttf_clip(clip: np.ndarray, H: int, W: int, r: int, t: float, anchor=None):
    """clip [F,N,C] float64.  Returns dict with anchor, best_sim[F,N], best_idx[F,N],
    fuse_map[F,N], src_index (output order) and pos [rows,3]."""
    F, N, C = clip.shape
    scores = anchor_scores(clip)
    a = int(np.argmax(scores)) if anchor is None else int(anchor) % F
    mask = window_mask(H, W, r)
    best_sim = np.ones((F, N))
    best_idx = np.tile(np.arange(N), (F, 1))
    fuse = np.full((F, N), -1, dtype=np.int64)
    thr = float(np.float32(t))
    for k in range(F):
        if k == a:
            continue
        s = np.where(mask, cos_matrix(clip[k], clip[a]), -np.inf)
        best_idx[k] = np.argmax(s, axis=1)
        best_sim[k] = s[np.arange(N), best_idx[k]]
        fused = best_sim[k] > thr
        fuse[k] = np.where(fused, best_idx[k], -1)
    keep = fuse < 0
    keep[a] = False
    flat_src = np.flatnonzero(keep.reshape(-1))
    src_index = np.concatenate([a * N + np.arange(N), flat_src])
    pos = np.stack([src_index // N, (src_index % N) // W, (src_index % N) % W], axis=1)
    return dict(anchor=a, scores=scores, best_sim=best_sim, best_idx=best_idx, fuse_map=fuse,
                src_index=src_index, pos=pos)


def ttf_tied(x: np.ndarray, H: int, W: int, r: int, t: float, anchor=None):
    """Tied-batch pass, x [B,F,N,C] float64: per candidate cell the mean over the batch of the
    cosines, arg max of the mean inside the window, every element's own cosine at that cell, and a
    position fused only if all elements exceed t.  Returns a dict like ttf_clip's."""
    B, F, N, C = x.shape
    scores = np.mean([anchor_scores(x[b]) for b in range(B)], axis=0)
    a = int(np.argmax(scores)) if anchor is None else int(anchor) % F
    mask = window_mask(H, W, r)
    thr = float(np.float32(t))
    mean_sim = np.ones((F, N))
    best_idx = np.tile(np.arange(N), (F, 1))
    best_sim = np.ones((B, F, N))
    fuse = np.full((F, N), -1, dtype=np.int64)
    for k in range(F):
        if k == a:
            continue
        s = np.stack([cos_matrix(x[b, k], x[b, a]) for b in range(B)])          # [B,N,N]
        m = np.where(mask, s.sum(axis=0) / B, -np.inf)
        best_idx[k] = np.argmax(m, axis=1)
        mean_sim[k] = m[np.arange(N), best_idx[k]]
        best_sim[:, k] = s[:, np.arange(N), best_idx[k]]
        fused = np.all(best_sim[:, k] > thr, axis=0)
        fuse[k] = np.where(fused, best_idx[k], -1)
    keep = fuse < 0
    keep[a] = False
    src_index = np.concatenate([a * N + np.arange(N), np.flatnonzero(keep.reshape(-1))])
    pos = np.stack([src_index // N, (src_index % N) // W, (src_index % N) % W], axis=1)
    return dict(anchor=a, scores=scores, mean_sim=mean_sim, best_sim=best_sim, best_idx=best_idx,
                fuse_map=fuse, src_index=src_index, pos=pos)
