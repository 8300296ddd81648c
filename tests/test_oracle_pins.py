"""Pins for the CPU oracle: each test checks it against something other than itself --
a second NumPy formulation, closed forms, textbook special cases, hand arithmetic, numbers
the paper prints -- so that a dropped term, wrong sign, wrong index or transposed operand in
the oracle fails at least one of them.  CPU only.
"""
import os

import numpy as np
import pytest

from workloads import CONFIGS, make_clip_batch, bf16_bits_to_f32, f32_to_bf16_bits
from workloads.ttf_gen import identical_frames, independent_frames, translated_frames

from bruteforce import anchor_scores, cos_matrix, ttf_clip, window_mask

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _table(name):
    rows = []
    with open(os.path.join(GOLD, name)) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([float(v) for v in line.split()])
    return rows


def _as_f64(x):
    return (bf16_bits_to_f32(x) if x.dtype == np.uint16 else x).astype(np.float64)


def _check_against_bruteforce(oracle, x, r, t, anchor_mode=0, anchor_index=0):
    B, F, H, W, C = x.shape
    N = H * W
    res = oracle.compress(x, r, t, anchor_mode, anchor_index)
    x64 = _as_f64(x).reshape(B, F, N, C)
    row = 0
    for b in range(B):
        ref = ttf_clip(x64[b], H, W, r, t, anchor=None if anchor_mode == 0 else anchor_index)
        assert res.anchor_index[b] == ref["anchor"]
        if anchor_mode == 0:
            np.testing.assert_allclose(res.anchor_score[b], ref["scores"], rtol=0, atol=1e-12)
        np.testing.assert_array_equal(res.best_idx[b], ref["best_idx"])
        np.testing.assert_allclose(res.best_sim[b], ref["best_sim"], rtol=0, atol=1e-12)
        np.testing.assert_array_equal(res.fuse_map[b], ref["fuse_map"])
        n = len(ref["src_index"])
        assert res.row_offsets[b] == row and res.kept_count[b] == n
        np.testing.assert_array_equal(res.src_index[row:row + n], ref["src_index"])
        np.testing.assert_array_equal(res.pos_ids[:, row:row + n].T, ref["pos"])
        row += n
    assert res.row_offsets[B] == row
    return res


# ---------------------------------------------------------------- whole pipeline vs brute force
def test_tiny_config_matches_bruteforce(oracle):
    cfg = CONFIGS["tiny"]
    batch = make_clip_batch(cfg)
    res = _check_against_bruteforce(oracle, batch.x, cfg.r, cfg.t[0])
    assert 0 < res.fused_fraction() < 1       # the case exercises both branches of the gate


@pytest.mark.parametrize("r", [0, 1, 2, 3])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_small_batches_match_bruteforce(oracle, r, dtype):
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=3, F=5, H=6, W=7, C=48, dtype=dtype, max_offset=min(r, 2) or 1)
    batch = make_clip_batch(cfg, seed=11 + r)
    _check_against_bruteforce(oracle, batch.x, r, 0.70)
    _check_against_bruteforce(oracle, batch.x, r, 0.70, anchor_mode=1, anchor_index=-1)
    _check_against_bruteforce(oracle, batch.x, r, 0.70, anchor_mode=1, anchor_index=2)


# ---------------------------------------------------------------- window search special cases
def test_full_grid_radius_is_global_matching(oracle):
    """r >= max(H,W)-1 makes the window the whole anchor grid: the global (F-1) N^2 matching
    of the introduction, i.e. the row-max of a normalised matrix product."""
    cfg = CONFIGS["tiny"].scaled(F=3, H=5, W=4, C=32)
    x = make_clip_batch(cfg, seed=5).x
    res = oracle.compress(x, max(cfg.H, cfg.W) - 1, 0.7, 1, 0)
    x64 = x.astype(np.float64).reshape(cfg.F, cfg.N, cfg.C)
    for k in range(1, cfg.F):
        s = cos_matrix(x64[k], x64[0])
        np.testing.assert_array_equal(res.best_idx[0, k], s.argmax(axis=1))
        np.testing.assert_allclose(res.best_sim[0, k], s.max(axis=1), atol=1e-12)
        assert (res.cand_count[0, k] == cfg.N).all()
    # a larger radius changes nothing
    res2 = oracle.compress(x, 50, 0.7, 1, 0)
    np.testing.assert_array_equal(res.best_idx, res2.best_idx)
    np.testing.assert_array_equal(res.best_sim, res2.best_sim)


def test_radius_zero_is_same_position_cosine(oracle):
    """The 1x1 window assumes zero motion (Section 4.3 A3): s^ is the cosine with the anchor
    token at the same cell and dst = i."""
    cfg = CONFIGS["tiny"].scaled(F=4, H=4, W=6, C=40)
    x = make_clip_batch(cfg, seed=8).x
    res = oracle.compress(x, 0, 0.7, 1, 1)
    x64 = x.astype(np.float64).reshape(cfg.F, cfg.N, cfg.C)
    a = x64[1]
    for k in (0, 2, 3):
        s = (x64[k] * a).sum(1) / (np.linalg.norm(x64[k], axis=1) * np.linalg.norm(a, axis=1))
        np.testing.assert_allclose(res.best_sim[0, k], s, atol=1e-12)
        np.testing.assert_array_equal(res.best_idx[0, k], np.arange(cfg.N))
        assert (res.cand_count[0, k] == 1).all()
        assert np.isneginf(res.second_sim[0, k]).all()


@pytest.mark.parametrize("H,W,r,per_frame", [(16, 16, 1, 2116), (8, 8, 1, 484), (32, 32, 2, 23716),
                                              (16, 16, 0, 256), (3, 5, 2, None)])
def test_candidate_counts(oracle, H, W, r, per_frame):
    """Distinct candidates after border-duplicate masking: product over the two axes of
    sum_z |[z-r, z+r] intersected with the axis|; interior tokens have (2r+1)^2 (Section 3)."""
    x = np.random.default_rng(0).standard_normal((1, 2, H, W, 2)).astype(np.float32)
    res = oracle.compress(x, r, 0.7, 1, 0)
    cnt = res.cand_count[0, 1].reshape(H, W)
    ax = lambda n: np.array([min(n - 1, z + r) - max(0, z - r) + 1 for z in range(n)])
    np.testing.assert_array_equal(cnt, ax(H)[:, None] * ax(W)[None, :])
    assert cnt.sum() == ax(H).sum() * ax(W).sum()
    if per_frame is not None:
        assert cnt.sum() == per_frame
    if H > 2 * r and W > 2 * r:
        assert (cnt[r:H - r, r:W - r] == (2 * r + 1) ** 2).all()
        assert cnt[0, 0] == (r + 1) ** 2
    assert (res.cand_count[0, 0] == 0).all()


def test_paper_cost_figures():
    """Numbers the paper prints: matching cost 18 / 164 / 456 MFLOPs for 1x1 / 3x3 / 5x5 scales
    as the (2r+1)^2 candidates per source token of its O((2r+1)^2 F N C) cost, and the avoided
    global matching is (F-1) N^2 > 2e6 inner products for F=32, N=256."""
    rows = _table("tab_window_mflops.txt")
    base = rows[0][2]
    for r, side, mflops in rows:
        assert side == 2 * r + 1
        lo, hi = (mflops - 0.5) / (base + 0.5), (mflops + 0.5) / (base - 0.5)
        assert lo <= (2 * r + 1) ** 2 <= hi
    F, N, bound = _table("global_matching_count.txt")[0]
    assert (F - 1) * N * N == 2031616 > bound
    # local matching at the default window evaluates (F-1) N (2r+1)^2 = 71424 candidate slots
    assert (F - 1) * N * 9 == 71424


def test_hand_example(oracle):
    rows = _table("hand_example.txt")
    x = np.array([[[1, 0], [0, 1], [4, 3]], [[3, 4], [0, 2], [-1, 0]]], dtype=np.float32).reshape(1, 2, 1, 3, 2)
    res = oracle.compress(x, 1, 0.70, 1, 0)
    for tok, s, dst, fused in rows:
        tok = int(tok)
        assert res.best_sim[0, 1, tok] == pytest.approx(s, abs=1e-15)
        assert res.best_idx[0, 1, tok] == int(dst)
        assert res.fuse_map[0, 1, tok] == (int(dst) if fused else -1)
    assert res.kept_count[0] == 4 and res.total_rows == 4
    np.testing.assert_array_equal(res.src_index[:4], [0, 1, 2, 5])
    np.testing.assert_array_equal(res.pos_ids[:, :4], [[0, 0, 0, 1], [0, 0, 0, 0], [0, 1, 2, 2]])
    np.testing.assert_array_equal(res.tokens_out[:4], [[1, 0], [0, 1], [4, 3], [-1, 0]])
    assert res.reduction_ratio()[0] == pytest.approx(1 - 4 / 6)
    # same data, last frame as anchor (negative index): roles swap
    res = oracle.compress(x, 1, 0.70, 1, -1)
    assert res.anchor_index[0] == 1
    # a0=(1,0) vs {s0=(3,4), s1=(0,2)}: 0.6, 0 ; a1=(0,1) vs {s0,s1,s2}: 0.8, 1, 0 ; a2=(4,3) vs {s1,s2}: 0.6, -0.8
    np.testing.assert_allclose(res.best_sim[0, 0], [0.6, 1.0, 0.6], atol=1e-15)
    np.testing.assert_array_equal(res.best_idx[0, 0], [0, 1, 1])
    np.testing.assert_array_equal(res.fuse_map[0, 0], [-1, 1, -1])
    np.testing.assert_array_equal(res.src_index[:5], [3, 4, 5, 0, 2])
    np.testing.assert_array_equal(res.pos_ids[:, :5], [[1, 1, 1, 0, 0], [0, 0, 0, 0, 0], [0, 1, 2, 0, 2]])


def test_planted_translation_is_recovered(oracle):
    """A source frame that is the anchor frame moved by (dy,dx), |d| <= r: every token whose
    origin lies in the grid matches it with cosine 1 and dst = origin cell."""
    cfg = CONFIGS["tiny"].scaled(F=5, H=7, W=9, C=64)
    shifts = [(1, 0), (0, -1), (-1, 1), (1, 1)]
    x = translated_frames(cfg, shifts, seed=3)
    res = oracle.compress(x, 1, 0.999, 1, 0)
    ys, xs = np.divmod(np.arange(cfg.N), cfg.W)
    for k, (dy, dx) in enumerate(shifts, start=1):
        oy, ox = np.clip(ys - dy, 0, cfg.H - 1), np.clip(xs - dx, 0, cfg.W - 1)
        np.testing.assert_allclose(res.best_sim[0, k], 1.0, atol=1e-12)
        np.testing.assert_array_equal(res.best_idx[0, k], oy * cfg.W + ox)
    assert res.kept_count[0] == cfg.N                      # everything fused at t = 0.999
    # a shift of 2 cells is outside the 3x3 window but inside the 5x5 one
    x2 = translated_frames(cfg, [(2, -2)], seed=3)
    r1 = oracle.compress(x2, 1, 0.9, 1, 0)
    r2 = oracle.compress(x2, 2, 0.9, 1, 0)
    assert (r1.fuse_map[0, 1] >= 0).sum() < cfg.N // 2
    assert (r2.fuse_map[0, 1] >= 0).all()


# ---------------------------------------------------------------- gating
def test_identical_frames_fuse_everything(oracle):
    cfg = CONFIGS["tiny"].scaled(B=2, F=6, H=5, W=5, C=64)
    x = identical_frames(cfg, seed=1)
    res = oracle.compress(x, 1, 0.7, 1, 3)
    src = np.ones((cfg.B, cfg.F), bool)
    src[:, 3] = False
    np.testing.assert_allclose(res.best_sim[src], 1.0, atol=1e-12)
    assert (res.fuse_map[src] == np.arange(cfg.N)).all()
    assert (res.kept_count == cfg.N).all()
    np.testing.assert_allclose(res.reduction_ratio(), 1 - 1 / cfg.F)


def test_independent_frames_fuse_nothing(oracle):
    cfg = CONFIGS["tiny"].scaled(B=1, F=4, H=6, W=6, C=1024)
    res = oracle.compress(independent_frames(cfg, seed=2), 1, 0.7)
    assert (res.fuse_map == -1).all()
    assert res.kept_count[0] == cfg.F * cfg.N and res.reduction_ratio()[0] == 0
    src = np.ones(cfg.F, bool)
    src[res.anchor_index[0]] = False
    assert np.abs(res.best_sim[0, src]).max() < 6 / np.sqrt(cfg.C)


def test_threshold_is_strict_and_monotone(oracle):
    # cos((1,1,1,1),(1,0,0,0)) = 1/2 exactly: kept at t = 0.5 (s^ <= t), fused just below
    x = np.array([[1, 0, 0, 0], [1, 1, 1, 1]], dtype=np.float32).reshape(1, 2, 1, 1, 4)
    assert oracle.compress(x, 1, 0.5, 1, 0).fuse_map[0, 1, 0] == -1
    assert oracle.compress(x, 1, np.nextafter(np.float32(0.5), np.float32(0)), 1, 0).fuse_map[0, 1, 0] == 0
    cfg = CONFIGS["qwen3vl_2b"].scaled(F=6, H=8, W=8, C=128)
    x = make_clip_batch(cfg, seed=4).x
    prev = None
    for t in (0.9, 0.8, 0.7, 0.6, 0.3):
        fused = oracle.compress(x, 1, t, 1, 0).fuse_map >= 0
        if prev is not None:
            assert (fused | ~prev).all()        # fused set only grows as t falls (ablation A1)
        prev = fused


def test_larger_window_never_lowers_best_similarity(oracle):
    cfg = CONFIGS["highres_wide"].scaled(B=1, F=4, H=8, W=8, C=96)
    x = make_clip_batch(cfg, seed=6).x
    prev = None
    for r in (0, 1, 2, 3):
        res = oracle.compress(x, r, 0.7, 1, 0)
        if prev is not None:
            assert (res.best_sim >= prev.best_sim).all()     # nested windows (ablation A3)
            assert ((res.fuse_map >= 0) | ~(prev.fuse_map >= 0)).all()
        prev = res


def test_zero_norm_token_is_kept(oracle):
    cfg = CONFIGS["tiny"].scaled(F=2, H=3, W=3, C=16)
    x = identical_frames(cfg, seed=7)
    x[0, 1, 1, 1] = 0.0
    res = oracle.compress(x, 1, 0.0, 1, 0)
    assert res.best_sim[0, 1, 4] == 0.0 and res.fuse_map[0, 1, 4] == -1
    x = identical_frames(cfg, seed=7)
    x[0, 0, 1, 1] = 0.0               # zero anchor token: cosine with it is 0, neighbours still match
    res = oracle.compress(x, 0, 0.5, 1, 0)
    assert res.best_sim[0, 1, 4] == 0.0 and res.fuse_map[0, 1, 4] == -1


def test_argmax_tie_goes_to_lowest_anchor_index(oracle):
    cfg = CONFIGS["tiny"].scaled(F=2, H=3, W=3, C=8)
    x = identical_frames(cfg, seed=9)
    x[0, 0, :, :] = x[0, 0, 1, 1]           # every anchor token identical
    res = oracle.compress(x, 1, 0.5, 1, 0)
    ys, xs = np.divmod(np.arange(9), 3)
    np.testing.assert_array_equal(res.best_idx[0, 1], np.maximum(ys - 1, 0) * 3 + np.maximum(xs - 1, 0))
    # two equal best candidates at (0,2) and (1,0) around the centre token: flat index 2 < 3 wins,
    # although (1,0) comes first in a column-major walk of the window
    x = identical_frames(cfg, seed=10)
    x[0, 0, 0, 2] = x[0, 1, 1, 1]
    x[0, 0, 1, 0] = x[0, 1, 1, 1]
    x[0, 0, 1, 1] = -x[0, 1, 1, 1]
    res = oracle.compress(x, 1, 0.5, 1, 0)
    assert res.best_idx[0, 1, 4] == 2 and res.best_sim[0, 1, 4] == pytest.approx(1.0, abs=1e-15)
    assert res.second_sim[0, 1, 4] == res.best_sim[0, 1, 4]      # the twin is the runner-up: a zero margin


# ---------------------------------------------------------------- compaction and positions
@pytest.mark.parametrize("name,scale", [("tiny", {}), ("qwen3vl_2b", dict(B=3, F=7, H=6, W=10, C=64)),
                                        ("long_video", dict(B=2, F=40, H=4, W=4, C=64, scene_len=8))])
def test_compaction_invariants(oracle, name, scale):
    cfg = CONFIGS[name].scaled(**scale)
    x = make_clip_batch(cfg).x
    res = oracle.compress(x, cfg.r, cfg.t[0])
    B, F, N, W = cfg.B, cfg.F, cfg.N, cfg.W
    rows = x.reshape(B, F * N, cfg.C)
    assert res.row_offsets[0] == 0 and res.total_rows == res.kept_count.sum()
    np.testing.assert_array_equal(np.diff(res.row_offsets), res.kept_count)
    for b in range(B):
        a = res.anchor_index[b]
        lo, hi = res.row_offsets[b], res.row_offsets[b + 1]
        src = res.src_index[lo:hi]
        fused = res.fuse_map[b] >= 0
        assert not fused[a].any()
        # kept + fused = F*N   and   L' = N + P
        assert (hi - lo) + fused.sum() == F * N
        assert res.kept_count[b] == N + (~fused).sum() - N
        np.testing.assert_array_equal(src[:N], a * N + np.arange(N))           # anchor rows first
        assert (np.diff(src[N:]) > 0).all()                                    # then ascending flat order
        assert not np.isin(src[N:] // N, a).any()
        np.testing.assert_array_equal(np.sort(src), np.flatnonzero(~fused.reshape(-1)))
        np.testing.assert_array_equal(res.pos_ids[:, lo:hi], [src // N, (src % N) // W, (src % N) % W])
        np.testing.assert_array_equal(res.tokens_out[lo:hi], rows[b][src])     # identity copy, no averaging
        assert ((res.fuse_map[b] >= 0) <= (res.fuse_map[b] == res.best_idx[b])).all()
        assert res.reduction_ratio()[b] == pytest.approx(1 - (hi - lo) / (F * N))
    assert (res.src_index[res.total_rows:] == -1).all()


def test_clips_are_independent(oracle):
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=3, F=5, H=4, W=4, C=32)
    x = make_clip_batch(cfg, seed=21).x
    whole = oracle.compress(x, 1, 0.7)
    for b in range(cfg.B):
        one = oracle.compress(x[b:b + 1], 1, 0.7)
        assert one.anchor_index[0] == whole.anchor_index[b]
        np.testing.assert_array_equal(one.fuse_map[0], whole.fuse_map[b])
        np.testing.assert_array_equal(one.best_sim[0], whole.best_sim[b])
        lo, hi = whole.row_offsets[b], whole.row_offsets[b + 1]
        np.testing.assert_array_equal(one.src_index[:hi - lo], whole.src_index[lo:hi])


def test_match_tokens_agrees_with_full_pass(oracle):
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=2, F=5, H=6, W=6, C=32)
    x = make_clip_batch(cfg, seed=22).x
    res = oracle.compress(x, 2, 0.7)
    rng = np.random.default_rng(0)
    tok = np.stack([rng.integers(0, cfg.B, 50), rng.integers(0, cfg.F, 50), rng.integers(0, cfg.N, 50)], 1)
    best, second, idx = oracle.match_tokens(x, 2, res.anchor_index, tok)
    np.testing.assert_array_equal(best, res.best_sim[tok[:, 0], tok[:, 1], tok[:, 2]])
    np.testing.assert_array_equal(second, res.second_sim[tok[:, 0], tok[:, 1], tok[:, 2]])
    np.testing.assert_array_equal(idx, res.best_idx[tok[:, 0], tok[:, 1], tok[:, 2]])


# ---------------------------------------------------------------- anchor rule
def test_anchor_hand_example(oracle):
    """F=3, N=1, C=2: tokens (1,0), (0,1), (1,1); clip mean (2/3,2/3); cosines 1/sqrt2, 1/sqrt2, 1."""
    x = np.array([[1, 0], [0, 1], [1, 1]], dtype=np.float32).reshape(1, 3, 1, 1, 2)
    res = oracle.compress(x, 1, 0.7)
    assert res.anchor_index[0] == 2
    np.testing.assert_allclose(res.anchor_score[0], [np.sqrt(0.5), np.sqrt(0.5), 1.0], atol=1e-15)
    # the mean is over raw tokens: scaling one frame's tokens changes the clip mean and the winner
    x = np.array([[10, 0], [0, 1], [1, 1]], dtype=np.float32).reshape(1, 3, 1, 1, 2)
    res = oracle.compress(x, 1, 0.7)
    g = np.array([11, 2]) / 3
    want = [11 / np.hypot(11, 2), 2 / np.hypot(11, 2), 13 / (np.sqrt(2) * np.hypot(11, 2))]
    np.testing.assert_allclose(res.anchor_score[0], want, atol=1e-15)
    assert res.anchor_index[0] == 0 and g[0] > g[1]


def test_anchor_uses_spatial_mean_not_single_tokens(oracle):
    """N=2: frame mean is the average of its two tokens."""
    x = np.array([[[2, 0], [0, 2]], [[3, 0], [1, 0]], [[0, 1], [0, 1]]], dtype=np.float32).reshape(1, 3, 1, 2, 2)
    res = oracle.compress(x, 0, 0.7)
    means = np.array([[1, 1], [2, 0], [0, 1]], dtype=np.float64)
    g = means.mean(0)
    want = means @ g / (np.linalg.norm(means, axis=1) * np.linalg.norm(g))
    np.testing.assert_allclose(res.anchor_score[0], want, atol=1e-15)
    assert res.anchor_index[0] == int(np.argmax(want)) == 0


def test_anchor_properties(oracle):
    cfg = CONFIGS["qwen3vl_2b"].scaled(F=9, H=4, W=5, C=96)
    batch = make_clip_batch(cfg, seed=31)
    x = batch.x
    res = oracle.compress(x, 1, 0.7)
    assert res.anchor_index[0] == batch.clean_frame[0, 0]      # the low-noise frame is the most representative
    np.testing.assert_allclose(res.anchor_score[0], anchor_scores(_as_f64(x)[0].reshape(cfg.F, cfg.N, cfg.C)), atol=1e-12)
    perm = np.random.default_rng(1).permutation(cfg.F)
    resp = oracle.compress(x[:, perm], 1, 0.7)
    np.testing.assert_allclose(resp.anchor_score[0], res.anchor_score[0][perm], atol=1e-12)
    assert perm[resp.anchor_index[0]] == res.anchor_index[0]
    dup = oracle.compress(np.concatenate([x, x], axis=1), 1, 0.7)   # duplicating the frames keeps every score
    np.testing.assert_allclose(dup.anchor_score[0][:cfg.F], res.anchor_score[0], atol=1e-12)
    assert dup.anchor_index[0] == res.anchor_index[0]               # and the tie goes to the lower index
    one = oracle.compress(x[:, :1], 1, 0.7)
    assert one.anchor_index[0] == 0 and one.kept_count[0] == cfg.N
    for fixed, want in ((0, 0), (-1, cfg.F - 1), (4, 4), (-cfg.F, 0)):
        assert oracle.compress(x, 1, 0.7, 1, fixed).anchor_index[0] == want
    with pytest.raises(ValueError):
        oracle.compress(x, 1, 0.7, 1, cfg.F)


def test_bf16_input_is_read_exactly(oracle):
    cfg = CONFIGS["tiny"].scaled(F=3, H=3, W=3, C=16)
    xf = make_clip_batch(cfg, seed=41).x
    bits = f32_to_bf16_bits(xf)
    a = oracle.compress(bits, 1, 0.7)
    b = oracle.compress(bf16_bits_to_f32(bits), 1, 0.7)
    np.testing.assert_array_equal(a.best_sim, b.best_sim)
    np.testing.assert_array_equal(a.src_index, b.src_index)
    assert a.tokens_out.dtype == np.uint16
    np.testing.assert_array_equal(bf16_bits_to_f32(a.tokens_out), b.tokens_out)
    # rounding is to nearest even: 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7 and goes to 1.0
    assert f32_to_bf16_bits(np.array([1 + 2.0 ** -8], np.float32))[0] == 0x3F80
    assert f32_to_bf16_bits(np.array([1 + 3 * 2.0 ** -8], np.float32))[0] == 0x3F82


def test_match_tokens_against_bruteforce(oracle):
    """The per-token entry point, pinned directly against the NumPy formulation (not via compress)."""
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=2, F=4, H=5, W=6, C=24, dtype="bf16")
    x = make_clip_batch(cfg, seed=23).x
    x64 = _as_f64(x).reshape(cfg.B, cfg.F, cfg.N, cfg.C)
    anchors = [1, 3]
    refs = [ttf_clip(x64[b], cfg.H, cfg.W, 2, 0.7, anchor=anchors[b]) for b in range(cfg.B)]
    tok = np.array([(b, k, i) for b in range(cfg.B) for k in range(cfg.F) for i in range(0, cfg.N, 3)])
    best, second, idx = oracle.match_tokens(x, 2, anchors, tok)
    for (b, k, i), s, j in zip(tok, best, idx):
        assert j == refs[b]["best_idx"][k, i]
        assert s == pytest.approx(refs[b]["best_sim"][k, i], abs=1e-12)
    src = tok[:, 1] != np.array(anchors)[tok[:, 0]]
    assert (second[src] <= best[src]).all() and np.isneginf(second[~src]).all()


def test_margin_helper_moves_every_decision_off_the_edge(oracle):
    from oracle import margins
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=2, F=6, H=8, W=8, C=64)
    batch = make_clip_batch(cfg, seed=24)
    before = oracle.compress(batch.x, 1, 0.7, want_tokens=False)
    ts = (0.7, 0.6)
    n_bad = len(margins.violators(before, ts, 5e-3, 1e-3))
    assert n_bad > 0                                   # wide margins: something has to move
    res = margins.enforce_margins(batch, 1, ts, sim_margin=5e-3, top2_margin=1e-3, want_tokens=False)
    assert len(margins.violators(res, ts, 5e-3, 1e-3)) == 0
    again = oracle.compress(batch.x, 1, 0.7, want_tokens=False)       # the batch was edited in place
    np.testing.assert_array_equal(again.fuse_map, res.fuse_map)
    src = np.ones_like(res.best_sim, bool)
    for b in range(cfg.B):
        src[b, res.anchor_index[b]] = False
    for t in ts:
        assert (np.abs(res.best_sim[src] - np.float32(t)) >= 5e-3).all()
    assert margins.anchor_gap(res) >= 1e-4


def test_tied_margin_helper_moves_every_decision_off_the_edge(oracle):
    from oracle import margins
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=3, F=5, H=6, W=6, C=32, dtype="bf16", shared_motion=True)
    batch = make_clip_batch(cfg)
    res = margins.enforce_tied_margins(batch, 1, (0.7,), want_tokens=False)
    src = np.ones(cfg.F, bool)
    src[res.anchor_index] = False
    assert np.all((res.mean_sim - res.second_mean)[src] >= 1e-4)
    assert np.all(np.abs(res.best_sim[:, src] - float(np.float32(0.7))) >= 1e-3)


def _random_small(n, seed):
    rng = np.random.default_rng(seed)
    return [(int(rng.integers(1, 4)), int(rng.integers(1, 7)), int(rng.integers(1, 8)), int(rng.integers(1, 10)),
             int(rng.choice([1, 3, 8, 24])), str(rng.choice(["f32", "bf16"])), int(rng.integers(0, 5)),
             float(rng.choice([0.2, 0.5, 0.7, 0.95]))) for _ in range(n)]


@pytest.mark.parametrize("B,F,H,W,C,dtype,r,t", _random_small(40, seed=11))
def test_random_small_problems_match_bruteforce(oracle, B, F, H, W, C, dtype, r, t):
    """Seeded sweep over odd little shapes (single rows and columns, one channel, radius beyond the
    grid, one frame): the plain pass and the tied-batch pass against their NumPy formulations."""
    from bruteforce import ttf_tied
    rng = np.random.default_rng(1000 * B + 100 * F + 10 * H + W + C + r)
    x = rng.standard_normal((B, F, H, W, C)).astype(np.float32)
    x[:, 1:] = 0.6 * x[:, 1:] + 0.8 * x[:, :1]                 # frames correlated with frame 0: both gate outcomes
    if dtype == "bf16":
        x = f32_to_bf16_bits(x)
    _check_against_bruteforce(oracle, x, r, t)
    res = oracle.compress_tied(x, r, t)
    ref = ttf_tied(_as_f64(x).reshape(B, F, H * W, C), H, W, r, t)
    assert res.anchor_index == ref["anchor"]
    np.testing.assert_array_equal(res.best_idx, ref["best_idx"])
    np.testing.assert_array_equal(res.fuse_map, ref["fuse_map"])
    np.testing.assert_allclose(res.best_sim, ref["best_sim"], rtol=0, atol=1e-12)
    assert res.kept_count == len(ref["src_index"])
    np.testing.assert_array_equal(res.src_index[:res.kept_count], ref["src_index"])


def test_nonfinite_entries_follow_ieee_arithmetic(oracle):
    """The similarity is the printed quotient evaluated in IEEE arithmetic: a source token with a NaN
    or infinite entry has a NaN cosine with every candidate, wins no comparison and is kept with
    s^ = -inf, dst = -1; an anchor token with such an entry is simply never the arg max.  Only an
    exactly zero norm gives cos = 0."""
    rng = np.random.default_rng(5)
    x = rng.standard_normal((1, 3, 4, 4, 16)).astype(np.float32)
    x[0, 1, 1, 1, 3] = np.nan          # source token 5 of frame 1
    x[0, 1, 2, 2, 0] = np.inf          # source token 10 of frame 1
    x[0, 2, 0, 0, :] = 0.0             # zero source token 0 of frame 2
    x[0, 0, 3, 3, 7] = -np.inf         # anchor token 15
    res = oracle.compress(x, 1, -0.5, 1, 0, want_tokens=False)      # anchor fixed to frame 0
    for i in (5, 10):
        assert res.best_sim[0, 1, i] == -np.inf and res.best_idx[0, 1, i] == -1 and res.fuse_map[0, 1, i] == -1
    assert res.best_sim[0, 2, 0] == 0.0 and res.fuse_map[0, 2, 0] >= 0          # cos = 0 > t = -0.5: fused
    assert (res.best_idx[0, 1:] != 15).all()                                    # the infinite anchor token never wins
    clean = np.delete(np.arange(16), [5, 10])
    assert np.isfinite(res.best_sim[0, 1, clean]).all()
