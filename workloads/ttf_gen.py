"""Seeded synthetic video-feature tensors shaped like a VLM's visual tokens.

The paper's clips are 32 frames of 16x16 merged tokens (8192 tokens, Introduction) whose
content reappears at almost the same grid cell in nearby frames (Introduction, "pointwise
temporal redundancy"), with one frame that is representative of the clip (Section 3, anchor
frame selection).  The recipes below keep exactly that structure and nothing else:

* ``chain``    every frame is the previous one moved by a per-region integer offset plus
               Gaussian noise, with a fraction of cells replaced by fresh content.
* ``anchored`` every frame is a latent scene moved by a per-region integer offset plus
               Gaussian noise whose amplitude varies per token, with a fraction of cells
               replaced by fresh content; one frame per scene is a low-noise copy of the
               scene.  Long clips are cut into scenes with independent latents.

Nothing here evaluates a similarity, picks an anchor or applies a threshold: this module
only draws numbers.  ``ClipBatch.redraw`` lets a caller that *has* judged tokens (the
margin helper that sits with the CPU oracle) replace single tokens with fresh draws.

bf16 tensors are carried as ``uint16`` bit patterns (NumPy has no bf16); rounding is
round-to-nearest-even from the fp32 value.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
from typing import Dict, Iterable, Optional, Sequence, Tuple

import numpy as np

_STREAM_META = 1    # offsets, clean-frame choice, amplitudes, scene-change mask
_STREAM_SCENE = 2   # latent scene content
_STREAM_NOISE = 3   # per-frame noise and fresh cells
_STREAM_REDRAW = 4  # single-token redraws


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    B: int
    F: int
    H: int
    W: int
    C: int
    dtype: str                    # "f32" or "bf16"
    r: int                        # search radius the workload is meant for
    t: Tuple[float, ...]          # threshold(s) the workload is meant for
    mode: str                     # "chain" or "anchored"
    max_offset: int               # per-region motion drawn from {-m..m}^2
    sigma: float                  # noise scale
    p_change: float               # fraction of cells replaced by fresh content
    seed: int
    region: int = 4               # motion offsets are constant on region x region cells
    scene_len: Optional[int] = None   # frames per scene (None: one scene per clip)
    clean_sigma: float = 0.3      # noise of the designated low-noise frame (anchored mode)
    shared_motion: bool = False   # every clip of the batch uses clip 0's motion, noise amplitudes, change mask
                                  # and low-noise frame (content and noise stay independent): views of one
                                  # scene dynamics, the input the tied-batch mode is meant for

    @property
    def N(self) -> int:
        return self.H * self.W

    @property
    def tokens(self) -> int:
        return self.B * self.F * self.H * self.W

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    def scaled(self, **kw) -> "WorkloadConfig":
        return replace(self, **kw)


# The five workloads, in the order the benchmark definition lists them.
CONFIGS: Dict[str, WorkloadConfig] = {
    "tiny": WorkloadConfig(
        "tiny", B=1, F=4, H=8, W=8, C=256, dtype="f32", r=1, t=(0.70,),
        mode="chain", max_offset=1, sigma=0.6, p_change=0.25, seed=1),
    "qwen3vl_2b": WorkloadConfig(
        "qwen3vl_2b", B=1, F=32, H=16, W=16, C=2048, dtype="bf16", r=1, t=(0.70,),
        mode="anchored", max_offset=1, sigma=0.628, p_change=0.10, seed=2),
    "qwen3vl_8b_batched": WorkloadConfig(
        "qwen3vl_8b_batched", B=16, F=32, H=16, W=16, C=4096, dtype="bf16", r=1, t=(0.70,),
        mode="anchored", max_offset=1, sigma=0.628, p_change=0.10, seed=3),
    "long_video": WorkloadConfig(
        "long_video", B=2, F=256, H=16, W=16, C=4096, dtype="bf16", r=1,
        t=(0.70, 0.60, 0.80),
        mode="anchored", max_offset=1, sigma=0.628, p_change=0.0, seed=4, scene_len=32),
    "highres_wide": WorkloadConfig(
        "highres_wide", B=4, F=64, H=32, W=32, C=4096, dtype="bf16", r=2, t=(0.70,),
        mode="anchored", max_offset=2, sigma=0.5, p_change=0.10, seed=5),
}


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(*key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(list(key)))


def _token_offsets(rng: np.random.Generator, cfg: WorkloadConfig) -> np.ndarray:
    """Per-token (oy, ox), constant on region x region blocks. Shape [H, W, 2]."""
    m = cfg.max_offset
    rh = -(-cfg.H // cfg.region)
    rw = -(-cfg.W // cfg.region)
    reg = rng.integers(-m, m + 1, size=(rh, rw, 2))
    full = np.repeat(np.repeat(reg, cfg.region, axis=0), cfg.region, axis=1)
    return full[: cfg.H, : cfg.W]


def _moved_coords(cfg: WorkloadConfig, off: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    yy, xx = np.meshgrid(np.arange(cfg.H), np.arange(cfg.W), indexing="ij")
    ys = np.clip(yy - off[..., 0], 0, cfg.H - 1)
    xs = np.clip(xx - off[..., 1], 0, cfg.W - 1)
    return ys, xs


def _scene_of(cfg: WorkloadConfig, k: int) -> int:
    return 0 if cfg.scene_len is None else k // cfg.scene_len


def _scene_latent(cfg: WorkloadConfig, seed: int, b: int, s: int) -> np.ndarray:
    return _rng(seed, b, _STREAM_SCENE, s).standard_normal((cfg.H, cfg.W, cfg.C), dtype=np.float32)


@dataclass
class ClipBatch:
    """A generated batch plus what is needed to redraw single tokens deterministically."""
    cfg: WorkloadConfig
    seed: int
    x: np.ndarray                  # [B,F,H,W,C] float32, or uint16 bf16 bit patterns
    offsets: np.ndarray            # [B,F,H,W,2] int8   motion applied to each token
    amplitude: np.ndarray          # [B,F,H,W]   float32 noise amplitude of each token
    changed: np.ndarray            # [B,F,H,W]   bool    cell was replaced by fresh content
    clean_frame: np.ndarray        # [B,n_scenes] int32  low-noise frame of each scene (-1: none)
    redraw_rounds: int = 0
    _latents: Dict[Tuple[int, int], np.ndarray] = field(default_factory=dict, repr=False)

    def as_f32(self, b: Optional[int] = None) -> np.ndarray:
        a = self.x if b is None else self.x[b]
        return bf16_bits_to_f32(a) if self.cfg.dtype == "bf16" else a

    def _store(self, b: int, k: int, y: int, xq: int, v: np.ndarray) -> None:
        if self.cfg.dtype == "bf16":
            self.x[b, k, y, xq] = f32_to_bf16_bits(v)
        else:
            self.x[b, k, y, xq] = v

    def redraw(self, tokens: Iterable[Tuple[int, int, int]], round_id: int) -> None:
        """Replace tokens (b, k, i) by fresh draws from the same recipe (unchanged motion)."""
        cfg = self.cfg
        for (b, k, i) in tokens:
            y, xq = divmod(int(i), cfg.W)
            rng = _rng(self.seed, int(b), _STREAM_REDRAW, int(k), int(i), int(round_id))
            oy, ox = (int(v) for v in self.offsets[b, k, y, xq])
            ys = min(max(y - oy, 0), cfg.H - 1)
            xs = min(max(xq - ox, 0), cfg.W - 1)
            if cfg.mode == "anchored":
                key = (int(b), _scene_of(cfg, int(k)))
                if key not in self._latents:
                    self._latents[key] = _scene_latent(cfg, self.seed, *key)
                base = self._latents[key][ys, xs]
                amp = np.float32(cfg.sigma * rng.uniform(0.0, 2.0))
            else:
                prev = self.as_f32(b)[k - 1, ys, xs] if k > 0 else self.as_f32(b)[0, y, xq]
                base = prev.astype(np.float32)
                amp = np.float32(cfg.sigma)
            eps = rng.standard_normal(cfg.C, dtype=np.float32)
            self._store(b, k, y, xq, base + amp * eps)
            self.amplitude[b, k, y, xq] = amp
            self.changed[b, k, y, xq] = False
        self.redraw_rounds = max(self.redraw_rounds, int(round_id) + 1)
        self._latents.clear()


def _emit(cfg: WorkloadConfig, frame: np.ndarray) -> np.ndarray:
    return f32_to_bf16_bits(frame) if cfg.dtype == "bf16" else frame.astype(np.float32, copy=False)


def _gen_clip(cfg: WorkloadConfig, seed: int, b: int, out: ClipBatch) -> None:
    meta = _rng(seed, 0 if cfg.shared_motion else b, _STREAM_META)
    H, W, C = cfg.H, cfg.W, cfg.C
    n_scenes = 1 if cfg.scene_len is None else -(-cfg.F // cfg.scene_len)
    if cfg.mode == "anchored":
        for s in range(n_scenes):
            k0 = 0 if cfg.scene_len is None else s * cfg.scene_len
            k1 = cfg.F if cfg.scene_len is None else min(cfg.F, k0 + cfg.scene_len)
            latent = _scene_latent(cfg, seed, b, s)
            kstar = k0 + int(meta.integers(0, k1 - k0))
            out.clean_frame[b, s] = kstar
            for k in range(k0, k1):
                noise = _rng(seed, b, _STREAM_NOISE, k)
                eps = noise.standard_normal((H, W, C), dtype=np.float32)
                if k == kstar:
                    off = np.zeros((H, W, 2), dtype=np.int64)
                    amp = np.full((H, W), cfg.clean_sigma, dtype=np.float32)
                    frame = latent + np.float32(cfg.clean_sigma) * eps
                    chg = np.zeros((H, W), dtype=bool)
                else:
                    off = _token_offsets(meta, cfg)
                    ys, xs = _moved_coords(cfg, off)
                    amp = (cfg.sigma * meta.uniform(0.0, 2.0, size=(H, W))).astype(np.float32)
                    frame = latent[ys, xs] + amp[..., None] * eps
                    chg = meta.random((H, W)) < cfg.p_change
                    if chg.any():
                        frame[chg] = noise.standard_normal((int(chg.sum()), C), dtype=np.float32)
                out.x[b, k] = _emit(cfg, frame)
                out.offsets[b, k] = off
                out.amplitude[b, k] = amp
                out.changed[b, k] = chg
    elif cfg.mode == "chain":
        out.clean_frame[b, :] = -1
        prev = _rng(seed, b, _STREAM_SCENE, 0).standard_normal((H, W, C), dtype=np.float32)
        out.x[b, 0] = _emit(cfg, prev)
        out.amplitude[b, 0] = 0.0
        for k in range(1, cfg.F):
            noise = _rng(seed, b, _STREAM_NOISE, k)
            off = _token_offsets(meta, cfg)
            ys, xs = _moved_coords(cfg, off)
            frame = prev[ys, xs] + np.float32(cfg.sigma) * noise.standard_normal((H, W, C), dtype=np.float32)
            chg = meta.random((H, W)) < cfg.p_change
            if chg.any():
                frame[chg] = noise.standard_normal((int(chg.sum()), C), dtype=np.float32)
            out.x[b, k] = _emit(cfg, frame)
            out.offsets[b, k] = off
            out.amplitude[b, k] = cfg.sigma
            out.changed[b, k] = chg
            prev = frame
    else:
        raise ValueError(f"unknown mode {cfg.mode!r}")


def make_clip_batch(cfg: WorkloadConfig, seed: Optional[int] = None, workers: int = 8) -> ClipBatch:
    """Generate one batch for ``cfg``. Clip ``b`` depends only on (seed, b)."""
    seed = cfg.seed if seed is None else int(seed)
    n_scenes = 1 if cfg.scene_len is None else -(-cfg.F // cfg.scene_len)
    shape = (cfg.B, cfg.F, cfg.H, cfg.W)
    out = ClipBatch(
        cfg=cfg, seed=seed,
        x=np.empty(shape + (cfg.C,), dtype=np.uint16 if cfg.dtype == "bf16" else np.float32),
        offsets=np.zeros(shape + (2,), dtype=np.int8),
        amplitude=np.zeros(shape, dtype=np.float32),
        changed=np.zeros(shape, dtype=bool),
        clean_frame=np.full((cfg.B, n_scenes), -1, dtype=np.int32),
    )
    workers = max(1, min(workers, cfg.B))
    if workers == 1:
        for b in range(cfg.B):
            _gen_clip(cfg, seed, b, out)
    else:
        with ThreadPoolExecutor(max_workers=workers) as pool:
            list(pool.map(lambda b: _gen_clip(cfg, seed, b, out), range(cfg.B)))
    return out


def identical_frames(cfg: WorkloadConfig, seed: int = 0) -> np.ndarray:
    """[B,F,H,W,C] where every frame of a clip equals its first frame (fp32 values)."""
    x = np.empty((cfg.B, cfg.F, cfg.H, cfg.W, cfg.C), dtype=np.float32)
    for b in range(cfg.B):
        f0 = _rng(seed, b, _STREAM_SCENE, 0).standard_normal((cfg.H, cfg.W, cfg.C), dtype=np.float32)
        x[b] = f0[None]
    return x


def independent_frames(cfg: WorkloadConfig, seed: int = 0) -> np.ndarray:
    """[B,F,H,W,C] of independent N(0,1) entries (fp32 values)."""
    return _rng(seed, 0, _STREAM_NOISE, 0).standard_normal(
        (cfg.B, cfg.F, cfg.H, cfg.W, cfg.C), dtype=np.float32)


def translated_frames(cfg: WorkloadConfig, shifts: Sequence[Tuple[int, int]], seed: int = 0) -> np.ndarray:
    """[1,F,H,W,C]: frame 0 is a random scene, frame k is frame 0 moved by shifts[k-1] with
    clamped borders (token (y,x) of frame k holds the content of (clamp(y-dy), clamp(x-dx)))."""
    f0 = _rng(seed, 0, _STREAM_SCENE, 0).standard_normal((cfg.H, cfg.W, cfg.C), dtype=np.float32)
    frames = [f0]
    for (dy, dx) in shifts:
        off = np.zeros((cfg.H, cfg.W, 2), dtype=np.int64)
        off[..., 0] = dy
        off[..., 1] = dx
        ys, xs = _moved_coords(cfg, off)
        frames.append(f0[ys, xs])
    return np.stack(frames)[None]


def similarity_field(B: int, F: int, N: int, seed: int = 0, ties: bool = False) -> Tuple[np.ndarray, np.ndarray]:
    """Stand-alone input for threshold selection: a float32 array [B,F,N] shaped like a field of
    best-match similarities (a fused mode near 0.9 and a changed mode near 0.35, clipped to
    [-1,1], a few exact zeros of either sign) and an int32 anchor frame per clip whose rows are set
    to 1.  With ``ties`` the values are rounded to two decimals so that many coincide."""
    rng = _rng(seed, _STREAM_META, 77)
    hi = rng.normal(0.9, 0.04, size=(B, F, N))
    lo = rng.normal(0.35, 0.15, size=(B, F, N))
    field = np.where(rng.random((B, F, N)) < 0.67, hi, lo).clip(-1.0, 1.0).astype(np.float32)
    if ties:
        field = np.round(field, 2).astype(np.float32)
    flat = field.reshape(-1)
    pick = rng.choice(flat.size, size=min(6, flat.size), replace=False)
    flat[pick[::2]] = np.float32(0.0)
    flat[pick[1::2]] = np.float32(-0.0)
    anchor = rng.integers(0, F, size=B).astype(np.int32)
    for b in range(B):
        field[b, anchor[b]] = 1.0
    return field, anchor
