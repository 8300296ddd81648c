"""GPU parity on inputs with NaN and +-Inf entries, in source frames and in the anchor frame, on every
search path.  The convention (include/ttf.h): values are not scanned; a candidate whose cosine is NaN
never wins the arg max; a source token none of whose candidates has a comparable cosine reports
best_sim = -inf, best_idx = -1 and is kept.  The oracle follows the same rule by construction
(comparisons with NaN are false), so every output must agree, NaN masks included."""
import numpy as np
import pytest

from workloads import CONFIGS, make_clip_batch, f32_to_bf16_bits
from workloads.ttf_gen import bf16_bits_to_f32

from helpers import compare_with_oracle, run_gpu

pytestmark = pytest.mark.gpu

ANCHOR_AUTO, ANCHOR_FIXED = 0, 1

PATHS = [
    # name,                 B, F,  H,  W,    C, dtype,  r, speculation
    ("matrix cores",        2, 5, 16, 16,  128, "bf16", 1, None),
    ("matrix cores 5x5",    1, 4, 16, 16,  256, "bf16", 2, None),
    ("padded tiles",        2, 4, 14, 14,  128, "bf16", 1, None),
    ("shared anchors",      2, 18, 64, 32, 128, "bf16", 2, None),
    ("speculative",         2, 6, 16, 16, 1024, "bf16", 1, 1),
    ("padded speculative",  2, 6, 14, 14, 1024, "bf16", 1, 1),
    ("ragged K-steps",      2, 5, 16, 16,   96, "bf16", 1, None),       # empty pass slots multiply zeros with anchor data
    ("padded ragged",       2, 4, 14, 14,   96, "bf16", 2, None),
    ("matrix cores fp32",   6, 5, 16, 16,  128, "f32",  1, None),       # a non-finite value makes its split pieces NaN
    ("padded fp32",         7, 4, 14, 14,   64, "f32",  2, None),
    ("general fp32",        2, 4,  6,  7,   33, "f32",  1, None),
    ("general bf16",        1, 4,  9,  9,   72, "bf16", 2, None),
    ("general tiled",       4, 33, 64, 16,  40, "f32",  1, None),
]


def _poison(x_f32, anchor, rng):
    """Plant non-finite entries: single elements and whole rows, in source frames and in frame `anchor`."""
    B, F, H, W, C = x_f32.shape
    src = [k for k in range(F) if k != anchor]
    planted = []

    def cell():
        return int(rng.integers(H)), int(rng.integers(W))

    for b in range(B):
        for value in (np.nan, np.inf, -np.inf):
            k = src[int(rng.integers(len(src)))]
            y, xq = cell()
            x_f32[b, k, y, xq, int(rng.integers(C))] = value            # one element of a source token
            planted.append((b, k, y * W + xq))
            y, xq = cell()
            x_f32[b, anchor, y, xq, int(rng.integers(C))] = value       # one element of an anchor token
        k = src[int(rng.integers(len(src)))]
        y, xq = cell()
        x_f32[b, k, y, xq, :] = np.nan                                  # a whole source row
        planted.append((b, k, y * W + xq))
        y, xq = cell()
        x_f32[b, anchor, y, xq, :] = np.inf                             # a whole anchor row
    return planted


@pytest.mark.parametrize("name,B,F,H,W,C,dtype,r,spec", PATHS, ids=[p[0] for p in PATHS])
@pytest.mark.parametrize("anchor", [1, "auto"])
def test_nonfinite_entries(oracle, name, B, F, H, W, C, dtype, r, spec, anchor):
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=B, F=F, H=H, W=W, C=C, dtype=dtype, r=r, max_offset=min(max(r, 1), 2),
                                       sigma=1.2, clean_sigma=0.1)
    from oracle import margins
    batch = make_clip_batch(cfg, seed=7000 + B + F + H + W + C + r)
    res0 = margins.enforce_margins(batch, r, (0.7,), want_tokens=False)     # clean decisions first
    x = bf16_bits_to_f32(batch.x).copy() if dtype == "bf16" else batch.x.copy()
    rng = np.random.default_rng(11 + C + F)
    if anchor == "auto":
        # non-finite entries in any frame make every anchor score NaN: the rule then falls to frame 0 on
        # both sides, so frame 0 is treated as the anchor when planting
        planted = _poison(x, 0, rng)
    else:
        planted = _poison(x, int(anchor), rng)
    x_in = f32_to_bf16_bits(x) if dtype == "bf16" else x
    mode, idx = (ANCHOR_AUTO, 0) if anchor == "auto" else (ANCHOR_FIXED, int(anchor))
    res = oracle.compress(x_in, r, 0.7, mode, idx, want_tokens=False)
    if anchor == "auto":
        assert (res.anchor_index == 0).all()
    # the planted source tokens have no comparable candidate: -inf / -1 / kept
    for (b, k, i) in planted:
        assert res.best_sim[b, k, i] == -np.inf and res.best_idx[b, k, i] == -1 and res.fuse_map[b, k, i] == -1
    assert res0.fused_fraction() > 0.05
    _, out = run_gpu(x_in, r, 0.7, anchor, speculation=spec)
    compare_with_oracle(x_in, out, res)
