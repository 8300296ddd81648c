"""GPU parity: the HIP library, called through its C ABI, against the fp64 CPU oracle on the
same seeded inputs.  Integer, index and byte outputs must match bit for bit; best_sim within
1e-5 absolute.  Inputs come from the workload generator with decision margins enforced
(|s^ - t| >= 1e-3, best - runner-up >= 1e-4, anchor score gap >= 1e-4), so that the fp32
GPU arithmetic and the fp64 oracle must take the same decisions."""
import numpy as np
import pytest
import torch

from workloads import CONFIGS, make_clip_batch, f32_to_bf16_bits
from workloads.ttf_gen import identical_frames, independent_frames, translated_frames

from helpers import compare_with_oracle, run_gpu, to_device

pytestmark = pytest.mark.gpu

ANCHOR_AUTO, ANCHOR_FIXED = 0, 1


def _prepared(cfg, seed=None, anchor="auto", ts=None, r=None):
    """Generate, enforce margins with the oracle, return (batch, oracle result for ts[0])."""
    from oracle import margins
    ts = cfg.t if ts is None else ts
    r = cfg.r if r is None else r
    mode, idx = (ANCHOR_AUTO, 0) if anchor == "auto" else (ANCHOR_FIXED, int(anchor))
    seed = cfg.seed if seed is None else seed
    for attempt in range(4):
        batch = make_clip_batch(cfg, seed=seed + 1000 * attempt)
        try:
            res = margins.enforce_margins(batch, r, ts, mode, idx, want_tokens=False)
            return batch, res
        except margins.MarginError:
            continue
    raise RuntimeError("no seed met the margins")


def _parity(cfg, seed=None, anchor="auto", r=None, t=None):
    r = cfg.r if r is None else r
    t = cfg.t[0] if t is None else t
    batch, res = _prepared(cfg, seed, anchor, ts=(t,), r=r)
    _, out = run_gpu(batch.x, r, t, anchor)
    compare_with_oracle(batch.x, out, res)
    return batch, res, out


# ----------------------------------------------------------------- the named workloads
def test_tiny_config():
    _, res, _ = _parity(CONFIGS["tiny"])
    assert 0 < res.fused_fraction() < 1


def test_qwen3vl_2b_config():
    _, res, _ = _parity(CONFIGS["qwen3vl_2b"])
    assert abs(res.fused_fraction() - 0.67) < 0.03


def test_qwen3vl_8b_batched_config():
    """The headline workload at full size, in the launch configuration the benchmark times."""
    _, res, _ = _parity(CONFIGS["qwen3vl_8b_batched"])
    assert abs(res.fused_fraction() - 0.67) < 0.02
    assert len(set(res.anchor_index.tolist())) > 4            # clips pick different anchors


def test_long_video_config_threshold_sweep(oracle):
    cfg = CONFIGS["long_video"]
    batch, res0 = _prepared(cfg)                               # margins hold for all three thresholds
    rhos = []
    for t in cfg.t:
        res = res0 if t == cfg.t[0] else oracle.compress(batch.x, cfg.r, t, want_tokens=False)
        _, out = run_gpu(batch.x, cfg.r, t)
        compare_with_oracle(batch.x, out, res)
        rhos.append(float(res.reduction_ratio().mean()))
    by_t = dict(zip(cfg.t, rhos))
    assert by_t[0.60] > by_t[0.70] > by_t[0.80] > 0.02         # lower threshold, more fusion (ablation A1)


def test_highres_wide_config():
    _, res, _ = _parity(CONFIGS["highres_wide"])
    assert res.fused_fraction() > 0.5


# ----------------------------------------------------------------- shapes that span tiles and ragged tails
F32_MFMA_SHAPES = [
    # fp32 tokens with whole 32-channel K-steps: matrix cores on three bf16 pieces per value (batch sizes
    # chosen so that the search has at least 48 workgroups: smaller problems take the general kernels)
    (6, 6, 16, 16, 256, "f32", 1),       # aligned 16-wide grid, two frames per wave
    (6, 5, 16, 16, 128, "f32", 2),       # 5x5 window: one frame per wave
    (6, 6, 16, 16, 96, "f32", 0),        # 1x1 window, 3 K-steps (one full round of the 3-deep pipeline)
    (6, 2, 16, 16, 32, "f32", 1),        # a single K-step and a single source frame
    (6, 3, 16, 16, 64, "f32", 1),        # two K-steps
    (6, 1, 16, 16, 128, "f32", 1),       # no source frame
    (3, 7, 8, 32, 128, "f32", 1),        # 32-wide grid
    (2, 4, 32, 32, 64, "f32", 2),        # 32-wide, 5x5 window
    (2, 18, 64, 32, 128, "f32", 2),      # 17 source frames: 4 full groups of 4 and one with a single frame
    (7, 6, 14, 14, 128, "f32", 1),       # padded tile rows
    (4, 4, 15, 20, 64, "f32", 2),        # odd height, second column tile partly empty
    (3, 5, 9, 40, 128, "f32", 1),        # wider than 32
    (4, 4, 6, 48, 32, "f32", 2),         # wide grid, 5x5 window: one workgroup per CU
    (3, 3, 4, 100, 64, "f32", 0),        # 7 column tiles
    (6, 6, 16, 16, 4096, "f32", 1),      # the full channel count (128 K-steps)
]

SHAPES = [
    # B, F, H,  W,  C,   dtype,  r
    (2, 3, 5, 7, 40, "f32", 1),          # N=35 < one 64-token word, C multiple of 4 only
    (1, 4, 9, 9, 33, "f32", 2),          # odd C: scalar loads
    (3, 5, 10, 13, 72, "bf16", 1),       # N=130: two full words and a ragged one
    (2, 4, 6, 6, 50, "bf16", 0),         # C % 8 != 0: scalar bf16 loads, 1x1 window
    (1, 6, 16, 16, 256, "bf16", 1),      # tile-aligned grid: matrix-core path, two K-steps per wave
    (2, 5, 16, 16, 128, "bf16", 2),      # matrix-core path, one K-step per wave, 5x5 window
    (1, 6, 16, 16, 384, "bf16", 0),      # matrix-core path, 1x1 window, last frame group partly empty
    (1, 2, 16, 16, 128, "bf16", 1),      # one source frame only
    (2, 1, 16, 16, 128, "bf16", 1),      # no source frame at all on the matrix-core path
    (3, 3, 4, 16, 512, "bf16", 1),       # N = 64: a single keep word per frame
    (2, 7, 8, 32, 128, "bf16", 1),       # 32-wide grid on the matrix-core path
    (1, 4, 32, 32, 256, "bf16", 2),      # 32-wide grid, 5x5 window
    (1, 5, 6, 32, 256, "bf16", 0),
    (2, 5, 16, 16, 96, "bf16", 2),
    (1, 3, 32, 32, 64, "bf16", 2),
    (1, 3, 32, 16, 128, "bf16", 3),
    (2, 3, 12, 20, 64, "f32", 30),       # radius beyond the grid: global matching
    (1, 2, 1, 1, 8, "f32", 1),           # single-token frames
    (1, 9, 3, 200, 32, "bf16", 1),       # wide, flat grid
    (2, 18, 64, 32, 128, "bf16", 2),     # 32-wide 5x5 with >= 512 workgroups: LDS-shared anchor kernel,
                                         # 17 source frames = 4 full groups of 4 and one group with one frame
    (1, 6, 512, 32, 128, "bf16", 2),     # same kernel on a tall grid, 5 source frames (second group: one frame)
    # grids up to 32 wide that are not 16 or 32 wide, or whose height leaves partial keep words: padded tile rows
    (2, 6, 14, 14, 128, "bf16", 1),      # 14x14: one padded column tile, N = 196
    (1, 11, 18, 24, 256, "bf16", 1),     # 24 wide: second column tile half empty; 10 source frames (two groups)
    (2, 4, 15, 20, 128, "bf16", 2),      # odd height, 5x5 window
    (1, 3, 27, 27, 128, "bf16", 0),      # 1x1 window
    (1, 5, 6, 16, 384, "bf16", 1),       # 16 wide but H % 4 != 0
    (2, 3, 5, 32, 128, "bf16", 2),       # 32 wide, odd height
    (1, 4, 3, 9, 128, "bf16", 1),        # fewer rows than a strip pair
    (1, 2, 1, 17, 128, "bf16", 2),       # a single grid row
    (3, 10, 7, 31, 128, "bf16", 1),
    # wider than 32: strips of 32 columns with the neighbouring column tiles on both sides
    (1, 5, 9, 40, 128, "bf16", 1),       # 3 column tiles, the last half empty; odd tile count
    (2, 4, 6, 48, 128, "bf16", 2),       # 5x5 window
    (1, 3, 4, 100, 256, "bf16", 0),      # 7 column tiles
    (1, 6, 5, 33, 128, "bf16", 1),       # one token in the third column tile
    (1, 4, 3, 64, 128, "bf16", 2),       # whole tiles only
    (2, 9, 20, 36, 128, "bf16", 1),
    (2, 1, 14, 14, 128, "bf16", 1),      # padded tile rows, no source frame
    (2, 6, 14, 14, 4096, "bf16", 1),     # padded and wide grids at the full channel count (128 K-steps)
    (1, 5, 10, 40, 4096, "bf16", 2),
    (1, 2, 70, 20, 1024, "bf16", 1),     # one source frame, long rows of channels (8 K-steps per pass variant not used here)
    (1, 3, 16, 16, 1024, "bf16", 1),     # fewer workgroups than CUs and C % 1024 == 0: one-frame long-pass variant
    (1, 5, 8, 32, 2048, "bf16", 2),      # the same variant on a 32-wide grid with a 5x5 window
    # channel counts that are whole 32-channel K-steps but do not divide over four waves or two-step passes
    (1, 4, 8, 32, 160, "bf16", 1),       # 5 K-steps: waves own 2, 2, 1 and 0 of them
    (2, 6, 16, 16, 4000, "bf16", 1),     # 125 K-steps: 32, 32, 32, 29
    (2, 5, 14, 14, 96, "bf16", 1),       # padded tile rows, 3 K-steps: the last pass half empty
    (1, 4, 6, 40, 224, "bf16", 2),       # wide grid, 7 K-steps, 5x5 window
    (1, 3, 12, 12, 32, "bf16", 2),       # a single K-step
    (4, 33, 384, 16, 32, "bf16", 1),     # 6144 workgroups: one wave walks every K-step, odd count (1)
    (2, 25, 128, 32, 96, "bf16", 2),     # the same on a 32-wide grid with a 5x5 window (3 K-steps)
    # general path at >= 2048 keep words: the LDS-tiled kernel (anchor halo staged per workgroup)
    (4, 33, 64, 16, 40, "f32", 1),       # fp32, one partial channel chunk
    (4, 33, 64, 16, 72, "bf16", 2),      # bf16 with C % 32 != 0, 5x5 window
    (4, 31, 63, 17, 264, "f32", 1),      # ragged keep words, two channel chunks
    (2, 40, 90, 20, 8, "bf16", 0),       # 1x1 window, a single 16-byte piece per row
    (3, 12, 64, 64, 16, "f32", 1),       # the LDS-tiled kernel on a 64-wide grid (eight patches per grid row)
    # whole 4 KiB slabs per row and at least 512 (frame, slab) pairs: the slab form of the frame sums
    (8, 32, 4, 4, 2048, "f32", 1),       # fp32, N = 16: two rounds of eight rows
    (4, 64, 3, 5, 4096, "bf16", 1),      # bf16, N = 15: one round and a tail of seven rows
    # long rows: ids first, then a copy driven by output rows
    (2, 4, 5, 7, 1536, "f32", 1),        # 6 KiB fp32 rows, N = 35: one ragged keep word, general path
    (1, 3, 9, 9, 3072, "bf16", 1),       # 6 KiB bf16 rows on padded tile rows
    (2, 3, 3, 70, 1540, "f32", 2),       # rows that are not a whole number of 256-piece rounds (385 pieces)
] + F32_MFMA_SHAPES


@pytest.mark.parametrize("B,F,H,W,C,dtype,r", SHAPES)
def test_shapes(B, F, H, W, C, dtype, r):
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=B, F=F, H=H, W=W, C=C, dtype=dtype, r=r, max_offset=min(max(r, 1), 2),
                                       sigma=0.5)
    _parity(cfg, seed=100 + B + F + H + W + C + r)


@pytest.mark.parametrize("anchor", [0, -1, 2, -3])
def test_fixed_anchor(anchor):
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=2, F=6, H=8, W=8, C=128)
    _, res, out = _parity(cfg, seed=7, anchor=anchor)
    assert (res.anchor_index == anchor % cfg.F).all()


# ----------------------------------------------------------------- degenerate cases
def _direct(x_np, r, t, anchor, oracle, check_sim=True):
    mode, idx = (ANCHOR_AUTO, 0) if anchor == "auto" else (ANCHOR_FIXED, int(anchor))
    res = oracle.compress(x_np, r, t, mode, idx, want_tokens=False)
    _, out = run_gpu(x_np, r, t, anchor)
    compare_with_oracle(x_np, out, res, check_sim=check_sim)
    return res, out


def test_single_frame(oracle):
    cfg = CONFIGS["tiny"].scaled(F=1)
    res, out = _direct(make_clip_batch(cfg).x, 1, 0.7, "auto", oracle)
    assert res.kept_count[0] == cfg.N


@pytest.mark.parametrize("C", [128, 1024])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_identical_frames_fuse_everything(oracle, dtype, C):
    """Every source token equals its anchor token: cos = 1 at dst = i, everything fused."""
    cfg = CONFIGS["tiny"].scaled(B=2, F=5, H=9, W=9, C=C)
    x = identical_frames(cfg, seed=3)
    x = f32_to_bf16_bits(x) if dtype == "bf16" else x
    res, out = _direct(x, 1, 0.7, 2, oracle)         # anchor fixed: all frame scores tie
    assert (res.kept_count == cfg.N).all()
    sim = out.buffers.best_sim.cpu().numpy()
    assert np.abs(sim - 1.0).max() <= 1e-5


def test_independent_frames_fuse_nothing(oracle):
    cfg = CONFIGS["tiny"].scaled(B=1, F=4, H=8, W=8, C=1024)
    res, _ = _direct(independent_frames(cfg, seed=4), 1, 0.7, 0, oracle)
    assert res.kept_count[0] == cfg.F * cfg.N


def test_translated_frames_recover_motion(oracle):
    cfg = CONFIGS["tiny"].scaled(F=5, H=7, W=9, C=64)
    x = translated_frames(cfg, [(1, 0), (0, -1), (-1, 1), (1, 1)], seed=5)
    # border tokens see the same content twice (clamped translation): ties between distinct anchor
    # tokens of equal similarity resolve to the lowest index on both sides
    res, _ = _direct(x, 1, 0.999, 0, oracle)
    assert res.kept_count[0] == cfg.N


def test_zero_rows(oracle):
    cfg = CONFIGS["tiny"].scaled(F=3, H=4, W=4, C=32)
    x = make_clip_batch(cfg, seed=6).x.copy()
    x[0, 1, 1, 1] = 0.0          # zero source token: cosine 0, kept
    x[0, 0, 2, 2] = 0.0          # zero anchor token
    res, out = _direct(x, 1, 0.0, 0, oracle)
    assert res.fuse_map[0, 1, 5] == -1 and out.buffers.best_sim[0, 1, 5].item() == 0.0


def test_duplicate_anchor_tokens_tie_to_lowest_index(oracle):
    cfg = CONFIGS["tiny"].scaled(F=2, H=6, W=6, C=64)
    x = identical_frames(cfg, seed=9)
    x[0, 0, :, :] = x[0, 0, 2, 2]
    res, _ = _direct(x, 1, 0.5, 0, oracle)
    ys, xs = np.divmod(np.arange(cfg.N), cfg.W)
    np.testing.assert_array_equal(res.best_idx[0, 1], np.maximum(ys - 1, 0) * cfg.W + np.maximum(xs - 1, 0))


def test_two_calls_are_bit_identical():
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=2, F=8)
    x_np = make_clip_batch(cfg, seed=12).x
    _, a = run_gpu(x_np, 1, 0.7)
    _, b = run_gpu(x_np, 1, 0.7)
    for name in ("tokens_out", "pos_ids", "src_index", "row_offsets", "kept_count", "anchor_index",
                 "fuse_map", "best_idx"):
        ta, tb = getattr(a.buffers, name), getattr(b.buffers, name)
        assert torch.equal(ta.view(torch.uint8), tb.view(torch.uint8)), name
    assert torch.equal(a.buffers.best_sim.view(torch.int32), b.buffers.best_sim.view(torch.int32))


@pytest.mark.parametrize("t", [-1.0, 1.0])
@pytest.mark.parametrize("C", [96, 128])
def test_threshold_extremes(oracle, t, C):
    """t = -1 fuses every source token, t = 1 fuses none (general and matrix-core kernels)."""
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=2, F=5, C=C)
    res, _ = _direct(make_clip_batch(cfg, seed=14).x, 1, t, "auto", oracle)
    want = cfg.N if t < 0 else cfg.F * cfg.N
    assert (res.kept_count == want).all()


@pytest.mark.parametrize("H,W,C", [(8, 8, 64), (16, 16, 256)])
def test_optional_outputs_and_host_counts(oracle, H, W, C):
    import paper_2605_07355_amd as ttf
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=3, F=4, H=H, W=W, C=C)
    batch, res = _prepared(cfg, seed=13)
    x = to_device(batch.x)
    buf = ttf.TTFBuffers.allocate(cfg.B, cfg.F, cfg.H, cfg.W, cfg.C, x.dtype, x.device, want_sim=False,
                                  want_host_counts=True)
    buf.host_counts.fill_(-1)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    out = ttf.ttf_compress(x, r=1, t=0.7, buffers=buf, want_sim=False, stream=side)   # a non-default stream
    side.synchronize()
    np.testing.assert_array_equal(buf.host_counts[:cfg.B].numpy(), res.kept_count)
    np.testing.assert_array_equal(buf.host_counts[cfg.B:].numpy(), res.row_offsets)
    np.testing.assert_array_equal(buf.fuse_map.cpu().numpy(), res.fuse_map)
    np.testing.assert_array_equal(buf.src_index.cpu().numpy()[:res.total_rows], res.src_index[:res.total_rows])


def test_errors_touch_nothing():
    import paper_2605_07355_amd as ttf
    cfg = CONFIGS["tiny"]
    x = to_device(make_clip_batch(cfg).x)
    buf = ttf.TTFBuffers.allocate(cfg.B, cfg.F, cfg.H, cfg.W, cfg.C, x.dtype, x.device)
    buf.fuse_map.fill_(-7)
    with pytest.raises(ttf.TTFError) as e:
        ttf.ttf_compress(x, r=-1, t=0.7, buffers=buf)
    assert e.value.status == 1
    with pytest.raises(ttf.TTFError) as e:
        ttf.ttf_compress(x, r=1, t=float("nan"), buffers=buf)
    assert e.value.status == 1
    with pytest.raises(ttf.TTFError) as e:
        ttf.ttf_compress(x, r=1, t=0.7, anchor=cfg.F, buffers=buf)
    assert e.value.status == 1
    small = ttf.TTFBuffers.allocate(cfg.B, cfg.F, cfg.H, cfg.W, cfg.C, x.dtype, x.device)
    small.workspace = small.workspace[:512]
    with pytest.raises(ttf.TTFError) as e:
        ttf.ttf_compress(x, r=1, t=0.7, buffers=small)
    assert e.value.status == 3
    torch.cuda.synchronize()
    assert (buf.fuse_map == -7).all()


def test_stage_profile_reports_every_stage():
    import paper_2605_07355_amd as ttf
    cfg = CONFIGS["qwen3vl_2b"].scaled(F=8)
    x = to_device(make_clip_batch(cfg).x)
    ttf.ttf_profile_enable(2)
    try:
        for _ in range(3):
            ttf.ttf_compress(x)
        ms = ttf.ttf_profile_read(2)
        ttf.ttf_profile_read(1)
        with pytest.raises(ttf.TTFError):
            ttf.ttf_profile_read(0)              # overwritten: only the last two calls are held
    finally:
        ttf.ttf_profile_enable(0)
    assert set(ms) == set(ttf.STAGE_NAMES)
    assert all(v >= 0 for v in ms.values()) and ms["window_search"] > 0


GRAPH_CASES = [
    # name,                      B, F,  H,  W,    C, dtype,  r, speculation
    ("aligned matrix cores",     2, 6, 16, 16,  256, "bf16", 1, None),
    ("padded tile rows",         2, 6, 14, 14,  128, "bf16", 1, None),       # dynamic LDS, k_pack_keep
    ("5x5 shared anchors",       2, 18, 64, 32, 128, "bf16", 2, None),       # dynamic LDS
    ("fp32 matrix cores",        6, 6, 16, 16,  128, "f32",  1, None),       # dynamic LDS
    ("fp32 padded tile rows",    7, 5, 14, 14,   64, "f32",  2, None),       # dynamic LDS, k_pack_keep
    ("general LDS-tiled",        4, 33, 64, 16,  40, "f32",  1, None),       # dynamic LDS
    ("speculative anchor route", 2, 6, 16, 16, 1024, "bf16", 1, 1),
    ("speculative, padded rows", 2, 6, 14, 14, 1024, "bf16", 1, 1),           # k_pack_keep after the second search
]


@pytest.mark.parametrize("name,B,F,H,W,C,dtype,r,spec", GRAPH_CASES, ids=[c[0] for c in GRAPH_CASES])
def test_graph_capture_and_replay(name, B, F, H, W, C, dtype, r, spec):
    """The call only enqueues kernels on the caller's stream (no allocation, no synchronisation), so
    it can be captured into a HIP graph.  Replays on new input contents, with eager work and
    synchronisations in between, must give what an eager call gives on the same contents."""
    import paper_2605_07355_amd as ttf
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=B, F=F, H=H, W=W, C=C, dtype=dtype, r=r, max_offset=min(max(r, 1), 2))
    xs = [to_device(make_clip_batch(cfg, seed=900 + i).x) for i in range(3)]
    x = torch.empty_like(xs[0])
    buf = ttf.TTFBuffers.allocate(B, F, H, W, C, x.dtype, x.device)
    ref = ttf.TTFBuffers.allocate(B, F, H, W, C, x.dtype, x.device)
    if spec is not None:
        ttf.ttf_set_speculation(spec)
    try:
        x.copy_(xs[0])
        ttf.ttf_compress(x, r=r, t=0.7, buffers=buf)                  # warm-up outside the capture
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            ttf.ttf_compress(x, r=r, t=0.7, buffers=buf)
        for i in (1, 2, 0, 1):
            x.copy_(xs[i])
            graph.replay()
            torch.cuda.synchronize()
            ttf.ttf_compress(xs[i], r=r, t=0.7, buffers=ref)          # eager, separate buffers
            torch.cuda.synchronize()
            rows = int(ref.row_offsets[-1])
            assert int(buf.row_offsets[-1]) == rows
            for field in ("anchor_index", "fuse_map", "kept_count", "row_offsets", "best_idx", "best_sim"):
                assert torch.equal(getattr(buf, field), getattr(ref, field)), field
            assert torch.equal(buf.src_index[:rows], ref.src_index[:rows])
            assert torch.equal(buf.pos_ids[:, :rows], ref.pos_ids[:, :rows])
            bits = torch.int16 if x.dtype == torch.bfloat16 else torch.int32
            assert torch.equal(buf.tokens_out[:rows].view(bits), ref.tokens_out[:rows].view(bits))
    finally:
        if spec is not None:
            ttf.ttf_set_speculation(0)


def _random_shapes(n, seed):
    """Seeded draw of small problems that spreads over every search path: grid widths around the
    tile boundaries (15..17, 31..33, 47..49), heights 1..12, radii 0..2 (3 now and then), channel
    counts that do and do not qualify for the matrix cores, both element types."""
    rng = np.random.default_rng(seed)
    widths = [1, 2, 7, 15, 16, 17, 24, 31, 32, 33, 40, 47, 48, 49, 65]
    out = []
    for _ in range(n):
        W = int(rng.choice(widths))
        H = int(rng.integers(1, 13))
        r = int(rng.choice([0, 1, 1, 2, 2, 3]))
        C = int(rng.choice([128, 128, 256, 384, 64, 100]))
        dtype = "bf16" if rng.random() < 0.8 else "f32"
        B = int(rng.integers(1, 4))
        F = int(rng.integers(1, 12))
        out.append((B, F, H, W, C, dtype, r))
    return out


@pytest.mark.parametrize("B,F,H,W,C,dtype,r", _random_shapes(36, seed=20260101))
def test_random_shapes(B, F, H, W, C, dtype, r):
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=B, F=F, H=H, W=W, C=C, dtype=dtype, r=r, max_offset=min(max(r, 1), 2),
                                       sigma=0.5, region=2)
    _parity(cfg, seed=500 + B + 3 * F + 5 * H + 7 * W + C + r)


# ----------------------------------------------------------------- inputs beyond 4 GiB
@pytest.mark.parametrize("name,kw,reps", [
    ("qwen3vl_8b_batched", dict(B=4), 20),                        # bf16, matrix-core path: 5 GiB in, B = 80
    ("qwen3vl_8b_batched", dict(B=4, C=1000, dtype="f32"), 36),   # fp32, general path: 4.4 GiB in, B = 144
])
def test_inputs_beyond_4gib(name, kw, reps):
    """Byte offsets past 2^32 in the input, the output and the workspace.  Clips are independent,
    so a batch made of `reps` copies of a small batch that agrees with the oracle must reproduce
    that small batch's outputs, clip for clip and bit for bit, at the shifted row offsets."""
    import paper_2605_07355_amd as ttf
    cfg = CONFIGS[name].scaled(**kw)
    batch, res, small = _parity(cfg)
    sb = small.buffers
    total = int(res.total_rows)
    x = to_device(batch.x)
    big_x = x.repeat(reps, 1, 1, 1, 1).contiguous()
    assert big_x.numel() * big_x.element_size() > (1 << 32)
    del x
    out = ttf.ttf_compress(big_x, r=cfg.r, t=cfg.t[0])
    torch.cuda.synchronize()
    bb = out.buffers
    B = cfg.B
    for got, want in ((bb.anchor_index, sb.anchor_index), (bb.kept_count, sb.kept_count),
                      (bb.fuse_map, sb.fuse_map), (bb.best_idx, sb.best_idx)):
        assert torch.equal(got.view(reps, *want.shape), want.unsqueeze(0).expand(reps, *want.shape))
    assert torch.equal(bb.best_sim.view(reps, *sb.best_sim.shape).view(torch.int32),
                       sb.best_sim.view(torch.int32).unsqueeze(0).expand(reps, *sb.best_sim.shape))
    offs = bb.row_offsets.cpu().numpy().astype(np.int64)
    want_offs = (np.arange(reps)[:, None] * total + res.row_offsets[None, :B]).reshape(-1)
    np.testing.assert_array_equal(offs[:-1], want_offs)
    assert offs[-1] == reps * total
    assert torch.equal(bb.src_index[:reps * total].view(reps, total), sb.src_index[:total].expand(reps, total))
    assert torch.equal(bb.pos_ids[:, :reps * total].view(3, reps, total),
                       sb.pos_ids[:, :total].unsqueeze(1).expand(3, reps, total))
    rows_small = sb.tokens_out.view(-1, cfg.C)[:total]
    rows_big = bb.tokens_out.view(-1, cfg.C)[:reps * total].view(reps, total, cfg.C)
    bits = torch.int16 if rows_small.dtype == torch.bfloat16 else torch.int32
    for rep in range(reps):
        assert torch.equal(rows_big[rep].view(bits), rows_small.view(bits)), f"copy {rep}"
