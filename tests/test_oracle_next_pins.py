"""Pins for the oracle's restoration, decode-alignment, adaptive-threshold and streaming-segment
functions, each against something other than itself: hand arithmetic, a second NumPy
formulation written from first principles, closed forms and library order statistics.  CPU only.
"""
import os

import numpy as np
import pytest

from workloads import CONFIGS, make_clip_batch, bf16_bits_to_f32
from workloads.ttf_gen import identical_frames, independent_frames

from bruteforce import ttf_clip

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _as_f64(x):
    return (bf16_bits_to_f32(x) if x.dtype == np.uint16 else x).astype(np.float64)


def _small(dtype="f32", seed=5, **kw):
    cfg = CONFIGS["tiny"].scaled(**{**dict(B=2, F=5, H=5, W=6, C=24, dtype=dtype, seed=seed), **kw})
    return cfg, make_clip_batch(cfg)


# ------------------------------------------------------------------------------ restoration
def _restore_of(oracle, x, r, t, mode=0, anchor=0):
    from oracle import restore as R
    res = oracle.compress(x, r, t, mode, anchor)
    rmap = R.restore_map(res.fuse_map, res.anchor_index, res.row_offsets, res.src_index)
    return res, rmap, R.restore(res.tokens_out, rmap)


def test_restore_hand_example(oracle):
    """Hand example (tests/golden/hand_example.txt): rows a0,a1,a2,s2; s0 and s1 are fused into a1."""
    x = np.array([[[1, 0], [0, 1], [4, 3]], [[3, 4], [0, 2], [-1, 0]]], dtype=np.float32).reshape(1, 2, 1, 3, 2)
    res, rmap, full = _restore_of(oracle, x, 1, 0.70, 1, 0)
    with open(os.path.join(GOLD, "hand_example_restore.txt")) as fh:
        want = [[float(v) for v in ln.split()] for ln in fh if ln.strip() and not ln.startswith("#")]
    np.testing.assert_array_equal(rmap.reshape(-1), [int(w[0]) for w in want])
    np.testing.assert_array_equal(full.reshape(-1, 2), [[w[1], w[2]] for w in want])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("r", [0, 1, 2])
def test_restore_matches_first_principles(oracle, dtype, r):
    """Every position must hold: its own token if it is an anchor token or its best similarity
    is <= t, else the anchor token of largest cosine in its window -- evaluated by the NumPy
    brute force, which shares nothing with the oracle."""
    cfg, batch = _small(dtype)
    x = batch.x
    B, F, H, W, C = x.shape
    N = H * W
    t = 0.6
    res, rmap, full = _restore_of(oracle, x, r, t)
    x64 = _as_f64(x).reshape(B, F, N, C)
    got = _as_f64(full).reshape(B, F, N, C)
    nfused = 0
    for b in range(B):
        ref = ttf_clip(x64[b], H, W, r, t)
        a = ref["anchor"]
        for k in range(F):
            for i in range(N):
                j = ref["fuse_map"][k, i]
                want = x64[b, a, j] if (k != a and j >= 0) else x64[b, k, i]
                nfused += int(k != a and j >= 0)
                np.testing.assert_array_equal(got[b, k, i], want)
    assert 0 < nfused < B * (F - 1) * N          # the case exercises both branches


def test_restore_of_identical_frames_is_the_input(oracle):
    x = identical_frames(CONFIGS["tiny"].scaled(B=2, F=4, H=4, W=5, C=16, dtype="f32"), seed=3)
    res, rmap, full = _restore_of(oracle, x, 1, 0.5)
    assert res.total_rows == 2 * 20               # everything fused ...
    np.testing.assert_array_equal(full, x.reshape(2, 4, 20, 16))   # ... and nothing lost


def test_restore_map_is_a_bijection_when_nothing_fuses(oracle):
    x = independent_frames(CONFIGS["tiny"].scaled(B=2, F=4, H=4, W=5, C=32, dtype="f32"), seed=4)
    res, rmap, full = _restore_of(oracle, x, 1, 0.99)
    assert res.total_rows == x.shape[0] * 4 * 20
    np.testing.assert_array_equal(np.sort(rmap.reshape(-1)), np.arange(res.total_rows))
    np.testing.assert_array_equal(full, x.reshape(2, 4, 20, 32))


def test_restore_map_structure(oracle):
    cfg, batch = _small("bf16", seed=8)
    res, rmap, full = _restore_of(oracle, batch.x, 1, 0.6)
    B, F, N = res.fuse_map.shape
    for b in range(B):
        lo, hi = res.row_offsets[b], res.row_offsets[b + 1]
        a = res.anchor_index[b]
        assert rmap[b].min() >= lo and rmap[b].max() < hi            # never leaves the clip
        np.testing.assert_array_equal(rmap[b, a], lo + np.arange(N))   # anchor rows come first, in order
        fused = res.fuse_map[b] >= 0
        assert np.all(rmap[b][fused] < lo + N)                       # fused -> an anchor row
        kept = ~fused
        kept[a] = False
        np.testing.assert_array_equal(rmap[b][kept], lo + N + np.arange(kept.sum()))  # ascending flat order
        # a row is referenced by the token it was copied from
        rows = np.arange(lo, hi)
        np.testing.assert_array_equal(rmap[b].reshape(-1)[res.src_index[lo:hi]], rows)


def test_decode_alignment_follows_the_cache(oracle):
    """Simulate the cache: prefill stores one pair per visual row and per text token; every decode
    step attends to everything stored plus itself, then stores one more pair."""
    from oracle import restore as R
    for l_prime, T in [(4, 0), (256 + 37, 19), (1, 1)]:
        cache = list(range(l_prime)) + list(range(T))
        for step in range(5):
            l_pre, pos, mask = R.decode_alignment(l_prime, T, step)
            assert l_pre == l_prime + T
            assert pos == len(cache)            # next free position index
            assert mask == len(cache) + 1       # all cached pairs and the new token
            cache.append(pos)


# ------------------------------------------------------------------------ adaptive threshold
@pytest.mark.parametrize("fraction", [0.0, 0.1, 0.33, 0.5, 0.67, 0.9, 1.0])
def test_threshold_is_the_inverted_cdf_quantile(fraction):
    """NumPy's inverted-CDF quantile is the order statistic at ceil(q M); with q = 1 - phi it must
    agree with the sort-based rule (a different library routine)."""
    from oracle import adaptive as A
    rng = np.random.default_rng(11)
    sim = rng.uniform(-0.2, 1.0, size=(3, 6, 35))
    anchor = np.array([0, 5, 2], np.int32)
    t = A.select_threshold(sim, anchor, fraction)
    q = 1.0 - float(np.float32(fraction))
    for b in range(3):
        src = np.delete(sim[b], anchor[b], axis=0).reshape(-1)
        if q * src.size <= 1.0:
            want = src.min()                    # rank clamps to the first order statistic
        else:
            want = np.quantile(src, q, method="inverted_cdf")
        assert t[b] == want


@pytest.mark.parametrize("fraction", [0.0, 0.25, 0.67, 1.0])
def test_threshold_fuses_the_requested_share(fraction):
    from oracle import adaptive as A
    rng = np.random.default_rng(12)
    sim = rng.permutation(np.linspace(0.0, 1.0, 4 * 50)).reshape(1, 4, 50)   # all distinct
    sim = np.concatenate([np.ones((1, 1, 50)), sim], axis=1)                  # frame 0 = anchor
    t = A.select_threshold(sim, np.array([0], np.int32), fraction)
    M = 200
    fused = int((sim[0, 1:] > t[0]).sum())
    want = int(np.floor(float(np.float32(fraction)) * M))
    assert fused == min(want, M - 1)            # the order statistic itself is never fused
    # ties at the threshold only ever lower the count
    sim2 = np.round(sim, 1)
    t2 = A.select_threshold(sim2, np.array([0], np.int32), fraction)
    assert int((sim2[0, 1:] > t2[0]).sum()) <= want


def test_threshold_edge_cases():
    from oracle import adaptive as A
    sim = np.ones((2, 1, 9), np.float32)                       # F = 1: no source tokens
    np.testing.assert_array_equal(A.select_threshold(sim, np.zeros(2, np.int32), 0.5), [1.0, 1.0])
    sim = np.full((1, 3, 4), 0.25, np.float32)                 # constant: t is that constant, nothing fused
    t = A.select_threshold(sim, np.array([1], np.int32), 0.9)
    assert t[0] == np.float32(0.25) and t.dtype == np.float32
    assert A.rank_for_fraction(0.0, 10) == 10 and A.rank_for_fraction(1.0, 10) == 1
    assert A.rank_for_fraction(0.5, 10) == 5 and A.rank_for_fraction(0.55, 10) == 5   # ceil(4.5)


def test_compress_per_clip_equals_batched_pass_at_one_threshold(oracle):
    """With the same t for every clip and the anchors the automatic rule picks, the per-clip
    assembly must reproduce the batched pass field by field."""
    from oracle import adaptive as A
    cfg, batch = _small("bf16", seed=21)
    ref = oracle.compress(batch.x, 1, 0.6)
    got = A.compress_per_clip(batch.x, 1, [0.6] * batch.x.shape[0], ref.anchor_index)
    for name in ("anchor_index", "best_idx", "fuse_map", "kept_count", "row_offsets", "src_index", "pos_ids",
                 "tokens_out", "best_sim"):
        np.testing.assert_array_equal(getattr(got, name), getattr(ref, name), err_msg=name)


def test_compress_per_clip_uses_each_clips_threshold(oracle):
    from oracle import adaptive as A
    cfg, batch = _small("f32", seed=22)
    x = batch.x
    B, F, H, W, C = x.shape
    ts = [0.3, 0.9]
    got = A.compress_per_clip(x, 1, ts, [0, 2])
    x64 = _as_f64(x).reshape(B, F, H * W, C)
    for b in range(B):
        ref = ttf_clip(x64[b], H, W, 1, ts[b], anchor=[0, 2][b])
        np.testing.assert_array_equal(got.fuse_map[b], ref["fuse_map"])
        lo, hi = got.row_offsets[b], got.row_offsets[b + 1]
        np.testing.assert_array_equal(got.src_index[lo:hi], ref["src_index"])
    assert got.kept_count[0] < got.kept_count[1]


# ------------------------------------------------------------------------ streaming segments
def test_segment_hand_example(oracle):
    """The hand example with its anchor frame handed in from outside: the three source tokens
    s0,s1 fuse, s2 is the only output row; temporal coordinate = frame_offset + 0."""
    from oracle import streaming as S
    anchor = np.array([[1, 0], [0, 1], [4, 3]], np.float32).reshape(1, 1, 3, 2)
    seg = np.array([[3, 4], [0, 2], [-1, 0]], np.float32).reshape(1, 1, 1, 3, 2)
    res = S.compress_segment(seg, anchor, 1, 0.70, frame_offset=7)
    np.testing.assert_allclose(res.best_sim[0, 0], [0.8, 1.0, 0.0], atol=1e-15)
    np.testing.assert_array_equal(res.fuse_map[0, 0], [1, 1, -1])
    assert res.total_rows == 1 and res.kept_count[0] == 1
    assert res.src_index[0] == 2
    np.testing.assert_array_equal(res.pos_ids[:, 0], [7, 0, 2])
    np.testing.assert_array_equal(res.tokens_out[0], [-1, 0])


def test_segment_matches_first_principles(oracle):
    """Brute force with the anchor frame prepended, re-indexed by hand."""
    from oracle import streaming as S
    cfg, batch = _small("bf16", seed=31, F=6)
    x = batch.x
    B, F, H, W, C = x.shape
    N = H * W
    anchor, seg = x[:, 0], x[:, 1:]
    res = S.compress_segment(seg, anchor, 1, 0.6, frame_offset=10)
    x64 = _as_f64(x).reshape(B, F, N, C)
    row = 0
    for b in range(B):
        ref = ttf_clip(x64[b], H, W, 1, 0.6, anchor=0)
        np.testing.assert_array_equal(res.fuse_map[b], ref["fuse_map"][1:])
        np.testing.assert_array_equal(res.best_idx[b], ref["best_idx"][1:])
        np.testing.assert_allclose(res.best_sim[b], ref["best_sim"][1:], rtol=0, atol=1e-12)
        kept = [(k, i) for k in range(1, F) for i in range(N) if ref["fuse_map"][k, i] < 0]
        assert res.row_offsets[b] == row and res.kept_count[b] == len(kept)
        for n, (k, i) in enumerate(kept):
            assert res.src_index[row + n] == (k - 1) * N + i
            np.testing.assert_array_equal(res.pos_ids[:, row + n], [10 + k - 1, i // W, i % W])
            np.testing.assert_array_equal(res.tokens_out[row + n], x[b, k].reshape(N, C)[i])
        row += len(kept)
    assert res.total_rows == row


def test_rolling_segments_of_a_static_stream_emit_nothing(oracle):
    """A stream that repeats one frame: after the first frame every segment fuses completely, so
    the rolling-anchor chain appends no rows at all."""
    from oracle import streaming as S
    x = identical_frames(CONFIGS["tiny"].scaled(B=1, F=7, H=4, W=4, C=16, dtype="f32"), seed=9)
    anchor = x[:, 0]
    total = 0
    for s0 in (1, 3, 5):
        seg = x[:, s0:s0 + 2]
        res = S.compress_segment(seg, anchor, 1, 0.9, frame_offset=s0)
        total += res.total_rows
        anchor = seg[:, -1]
    assert total == 0


def test_one_frame_segments_with_rolling_anchor_are_frame_differencing(oracle):
    """Segments of one frame: frame k is matched against frame k-1 (not against a global anchor).
    Checked with the brute force on the two-frame clip [k-1, k]."""
    from oracle import streaming as S
    cfg, batch = _small("f32", seed=33, B=1, F=4)
    x = batch.x
    B, F, H, W, C = x.shape
    N = H * W
    x64 = _as_f64(x).reshape(B, F, N, C)
    for k in range(1, F):
        res = S.compress_segment(x[:, k:k + 1], x[:, k - 1], 1, 0.6, frame_offset=k)
        ref = ttf_clip(x64[0, k - 1:k + 1], H, W, 1, 0.6, anchor=0)
        np.testing.assert_array_equal(res.fuse_map[0, 0], ref["fuse_map"][1])
        assert np.all(res.pos_ids[0, :res.total_rows] == k)


# ------------------------------------------------------------------------------ tied batch
def _tied_cfg(**kw):
    return CONFIGS["qwen3vl_2b"].scaled(**{**dict(B=3, F=5, H=5, W=6, C=24, dtype="f32", seed=41,
                                                   shared_motion=True), **kw})


def test_tied_hand_example(oracle):
    with open(os.path.join(GOLD, "hand_example_tied.txt")) as fh:
        rows = [[float(v) for v in ln.split()] for ln in fh if ln.strip() and not ln.startswith("#")]
    e0 = [[[1, 0], [0, 1], [4, 3]], [[3, 4], [0, 2], [-1, 0]]]
    e1 = [[[1, 0], [0, 1], [3, 4]], [[1, 0], [3, 4], [0, -1]]]
    x = np.array([e0, e1], dtype=np.float32).reshape(2, 2, 1, 3, 2)
    res = oracle.compress_tied(x, 1, 0.70, 1, 0)
    for tok, dst, mean, s0, s1, fused in rows:
        tok = int(tok)
        assert res.best_idx[1, tok] == int(dst)
        assert res.mean_sim[1, tok] == pytest.approx(mean, abs=1e-15)
        assert res.best_sim[0, 1, tok] == pytest.approx(s0, abs=1e-15)
        assert res.best_sim[1, 1, tok] == pytest.approx(s1, abs=1e-15)
        assert res.fuse_map[1, tok] == (int(dst) if fused else -1)
    assert res.kept_count == 5
    np.testing.assert_array_equal(res.src_index[:5], [0, 1, 2, 3, 5])
    np.testing.assert_array_equal(res.pos_ids[:, :5], [[0, 0, 0, 1, 1], [0] * 5, [0, 1, 2, 0, 2]])
    np.testing.assert_array_equal(res.tokens_out[0, :5], [[1, 0], [0, 1], [4, 3], [3, 4], [-1, 0]])
    np.testing.assert_array_equal(res.tokens_out[1, :5], [[1, 0], [0, 1], [3, 4], [1, 0], [0, -1]])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("r", [0, 1, 2])
def test_tied_matches_bruteforce(oracle, dtype, r):
    from bruteforce import ttf_tied
    cfg = _tied_cfg(dtype=dtype)
    x = make_clip_batch(cfg).x
    B, F, H, W, C = x.shape
    N = H * W
    t = 0.55
    res = oracle.compress_tied(x, r, t)
    ref = ttf_tied(_as_f64(x).reshape(B, F, N, C), H, W, r, t)
    assert res.anchor_index == ref["anchor"]
    np.testing.assert_allclose(res.anchor_score, ref["scores"], rtol=0, atol=1e-12)
    np.testing.assert_array_equal(res.best_idx, ref["best_idx"])
    np.testing.assert_allclose(res.mean_sim, ref["mean_sim"], rtol=0, atol=1e-12)
    np.testing.assert_allclose(res.best_sim, ref["best_sim"], rtol=0, atol=1e-12)
    np.testing.assert_array_equal(res.fuse_map, ref["fuse_map"])
    n = len(ref["src_index"])
    assert res.kept_count == n
    np.testing.assert_array_equal(res.src_index[:n], ref["src_index"])
    np.testing.assert_array_equal(res.pos_ids[:, :n].T, ref["pos"])
    xin = x.reshape(B, F * N, C)
    for b in range(B):
        np.testing.assert_array_equal(res.tokens_out[b, :n], xin[b][ref["src_index"]])
    fused = (res.fuse_map >= 0).mean()
    assert 0.05 < fused < 0.95                      # both outcomes occur


def test_tied_with_one_element_is_the_plain_pass(oracle):
    cfg, batch = _small("bf16", seed=43, B=1)
    one = oracle.compress(batch.x, 1, 0.6)
    tied = oracle.compress_tied(batch.x, 1, 0.6)
    assert tied.anchor_index == one.anchor_index[0] and tied.kept_count == one.kept_count[0]
    np.testing.assert_array_equal(tied.fuse_map, one.fuse_map[0])
    np.testing.assert_array_equal(tied.best_idx, one.best_idx[0])
    np.testing.assert_array_equal(tied.best_sim[0], one.best_sim[0])
    np.testing.assert_array_equal(tied.mean_sim, one.best_sim[0])
    n = tied.kept_count
    np.testing.assert_array_equal(tied.src_index[:n], one.src_index[:n])
    np.testing.assert_array_equal(tied.tokens_out[0, :n], one.tokens_out[:n])


def test_tied_copies_of_one_clip_behave_like_that_clip(oracle):
    """B identical elements: the mean equals each element's similarity, so every decision is the
    single clip's and all elements emit the same rows."""
    cfg, batch = _small("f32", seed=44, B=1)
    x = np.repeat(batch.x, 3, axis=0)
    one = oracle.compress(batch.x, 2, 0.6)
    tied = oracle.compress_tied(x, 2, 0.6)
    np.testing.assert_array_equal(tied.fuse_map, one.fuse_map[0])
    np.testing.assert_allclose(tied.mean_sim, one.best_sim[0], rtol=0, atol=1e-15)
    for b in range(3):
        np.testing.assert_array_equal(tied.tokens_out[b, :tied.kept_count], one.tokens_out[:one.kept_count[0]])


def test_tied_union_rule_and_fixed_anchor(oracle):
    cfg = _tied_cfg(seed=45)
    x = make_clip_batch(cfg).x
    t = 0.6
    res = oracle.compress_tied(x, 1, t, 1, -1)
    assert res.anchor_index == cfg.F - 1
    src = np.ones(cfg.F, bool)
    src[res.anchor_index] = False
    fused = res.fuse_map >= 0
    above = np.all(res.best_sim > float(np.float32(t)), axis=0)
    np.testing.assert_array_equal(fused[src], above[src])        # fused iff every element exceeds t
    assert not fused[~src].any()
    # a position one element alone would fuse can still be kept because another element objects
    some = (res.best_sim > float(np.float32(t)))[:, src]
    assert (some.any(axis=0) & ~some.all(axis=0)).any()
    np.testing.assert_allclose(res.mean_sim[src] >= res.second_mean[src], True)


def test_tied_gate_is_strict_per_element(oracle):
    """cos((1,1,1,1),(1,0,0,0)) = 1/2 exactly.  At t = 1/2 that element is not above t, so the
    position is kept although the other element matches perfectly; just below 1/2 it fuses."""
    anchor = [[1, 0, 0, 0]]
    x = np.array([[anchor, [[1, 1, 1, 1]]], [anchor, [[1, 0, 0, 0]]]], np.float32).reshape(2, 2, 1, 1, 4)
    res = oracle.compress_tied(x, 0, 0.5, 1, 0)
    np.testing.assert_array_equal(res.best_sim[:, 1, 0], [0.5, 1.0])
    assert res.mean_sim[1, 0] == 0.75
    assert res.fuse_map[1, 0] == -1 and res.kept_count == 2
    res = oracle.compress_tied(x, 0, float(np.nextafter(np.float32(0.5), np.float32(0))), 1, 0)
    assert res.fuse_map[1, 0] == 0 and res.kept_count == 1


def test_tied_anchor_is_the_batch_mean_of_the_scores(oracle):
    """Two elements that disagree about the best frame: the shared anchor follows the mean score,
    checked against the single-clip scores of the already pinned plain pass."""
    cfg = _tied_cfg(seed=46, B=4, shared_motion=False)
    x = make_clip_batch(cfg).x
    per = oracle.compress(x, 1, 0.6, want_tokens=False)
    tied = oracle.compress_tied(x, 1, 0.6, want_tokens=False)
    mean = per.anchor_score.mean(axis=0)
    np.testing.assert_allclose(tied.anchor_score, mean, rtol=0, atol=1e-15)
    assert tied.anchor_index == int(np.argmax(mean))
    assert len(set(per.anchor_index.tolist())) > 1        # the elements alone would not agree


def test_tied_ties_go_to_the_lowest_index(oracle):
    """Equal batch-mean similarities at two anchor cells (the anchor frame repeats a token) and
    equal anchor scores (identical frames): the first maximum wins in both rules."""
    rng = np.random.default_rng(50)
    frame = rng.standard_normal((2, 1, 4, 8)).astype(np.float32)        # B=2, grid 1x4
    frame[:, 0, 2] = frame[:, 0, 1]                                     # cells 1 and 2 hold the same token
    x = np.repeat(frame[:, None], 3, axis=1)                            # three identical frames
    res = oracle.compress_tied(x, 1, 0.5)
    assert res.anchor_index == 0                                        # all frames score the same
    np.testing.assert_array_equal(res.best_idx[1], [0, 1, 1, 3])        # token 2 ties between cells 1 and 2
    np.testing.assert_array_equal(res.best_idx[2], [0, 1, 1, 3])
    assert res.second_mean[1, 2] == res.mean_sim[1, 2]                  # the twin is the runner-up
