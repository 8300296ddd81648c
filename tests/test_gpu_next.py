"""GPU parity of the follow-on entry points (restoration, decode alignment, adaptive threshold
and re-gating) against the oracle modules, through the C ABI.  Integer and byte outputs bit for
bit; a selected threshold is an order statistic of float32 inputs and must match exactly when
both sides are given the same array."""
import ctypes

import numpy as np
import pytest
import torch

from workloads import CONFIGS, make_clip_batch, similarity_field

from helpers import SENTINEL, compare_with_oracle, rows_as_bits, run_gpu, to_device

pytestmark = pytest.mark.gpu

ANCHOR_AUTO, ANCHOR_FIXED = 0, 1


def _prepared(cfg, ts, r=None):
    from oracle import margins
    r = cfg.r if r is None else r
    for attempt in range(4):
        batch = make_clip_batch(cfg, seed=cfg.seed + 1000 * attempt)
        try:
            return batch, margins.enforce_margins(batch, r, ts, ANCHOR_AUTO, 0, want_tokens=True)
        except margins.MarginError:
            continue
    raise RuntimeError("no seed met the margins")


SMALL = [
    ("tiny", {}),
    ("qwen3vl_2b", dict(B=2, F=5, H=14, W=14, C=128)),                 # matrix-core path on padded tile rows
    ("qwen3vl_2b", dict(B=2, F=6)),                                    # matrix-core search path, 16x16 grid
    ("tiny", dict(B=3, F=5, H=7, W=9, C=40, dtype="f32")),             # ragged keep words, scalar rows
    ("tiny", dict(B=2, F=4, H=5, W=13, C=129, dtype="bf16")),          # odd row length (2-byte copies)
    ("tiny", dict(B=2, F=4, H=5, W=7, C=1540, dtype="f32")),           # long rows: one block per token, 385 pieces
    ("qwen3vl_2b", dict(B=1, F=4, H=6, W=16, C=1024)),                 # 2 KiB rows: 128-thread blocks in restoration
    ("qwen3vl_2b", dict(B=6, F=5, C=128, dtype="f32")),                # fp32 tokens on the matrix cores
]


# ------------------------------------------------------------------------------ restoration
@pytest.mark.parametrize("name,scale", SMALL)
def test_restore_map_and_rows(name, scale):
    import paper_2605_07355_amd as ttf
    from oracle import restore as R
    cfg = CONFIGS[name].scaled(**scale)
    batch, res = _prepared(cfg, (cfg.t[0],))
    x, out = run_gpu(batch.x, cfg.r, cfg.t[0])
    compare_with_oracle(batch.x, out, res)
    want_map = R.restore_map(res.fuse_map, res.anchor_index, res.row_offsets, res.src_index)
    rmap = torch.full((cfg.B, cfg.F, cfg.H * cfg.W), SENTINEL, dtype=torch.int32, device="cuda")
    ttf.ttf_restore_map(out, rmap)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(rmap.cpu().numpy(), want_map)
    full = torch.empty_like(x)
    full.view(torch.uint8).fill_(0x5B)
    ttf.ttf_restore(out.buffers.tokens_out, res.total_rows, rmap, cfg.H, cfg.W, full)
    torch.cuda.synchronize()
    want = R.restore(res.tokens_out, want_map)                         # [B,F,N,C] in the input's bit type
    np.testing.assert_array_equal(rows_as_bits(full).reshape(want.shape),
                                  want.view(np.uint16 if want.dtype == np.uint16 else np.uint32))


def test_restore_at_full_size_by_property():
    """Headline workload: the map against the oracle's in full; the restored tensor through what
    it must equal at any size -- the input itself at retained positions, the matched anchor token
    at fused ones (indices taken from the oracle's fuse_map)."""
    import paper_2605_07355_amd as ttf
    from oracle import restore as R
    cfg = CONFIGS["qwen3vl_8b_batched"]
    batch, res = _prepared(cfg, (cfg.t[0],))
    x, out = run_gpu(batch.x, cfg.r, cfg.t[0])
    rmap = ttf.ttf_restore_map(out)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(rmap.cpu().numpy(),
                                  R.restore_map(res.fuse_map, res.anchor_index, res.row_offsets, res.src_index))
    full = ttf.ttf_restore(out.buffers.tokens_out, res.total_rows, rmap, cfg.H, cfg.W)
    torch.cuda.synchronize()
    B, F, N, C = cfg.B, cfg.F, cfg.H * cfg.W, cfg.C
    fm = torch.from_numpy(res.fuse_map).cuda().long()                  # [B,F,N]
    a = torch.from_numpy(res.anchor_index).cuda().long()
    xv = x.view(B, F, N, C).view(torch.int16)
    fv = full.view(B, F, N, C).view(torch.int16)
    for b in range(B):
        fused = fm[b] >= 0
        assert torch.equal(fv[b][~fused], xv[b][~fused])
        assert torch.equal(fv[b][fused], xv[b, a[b]][fm[b][fused]])


def test_restore_map_entries_outside_the_rows_give_zero_rows():
    import paper_2605_07355_amd as ttf
    tokens = torch.arange(6 * 8, dtype=torch.float32, device="cuda").view(6, 8) + 1.0
    rmap = torch.tensor([[[0, 5, -1, 6]]], dtype=torch.int32, device="cuda")       # B=1,F=1,N=4 ; rows = 6
    full = ttf.ttf_restore(tokens, 6, rmap, 2, 2)
    torch.cuda.synchronize()
    got = full.view(4, 8).cpu().numpy()
    np.testing.assert_array_equal(got[0], tokens[0].cpu().numpy())
    np.testing.assert_array_equal(got[1], tokens[5].cpu().numpy())
    assert (got[2] == 0).all() and (got[3] == 0).all()
    full = ttf.ttf_restore(tokens, 3, rmap, 2, 2)                      # fewer valid rows: entry 5 is now outside
    torch.cuda.synchronize()
    assert (full.view(4, 8)[1] == 0).all()


def test_decode_alignment_matches_the_oracle():
    import paper_2605_07355_amd as ttf
    from oracle import restore as R
    for args in [(0, 0, 0), (256 + 91, 33, 0), (256 + 91, 33, 17), (2 ** 31, 2 ** 20, 5)]:
        assert ttf.ttf_decode_alignment(*args) == R.decode_alignment(*args)
    with pytest.raises(ttf.TTFError):
        ttf.ttf_decode_alignment(-1, 0, 0)


# ------------------------------------------------------------------------ adaptive threshold
class _FakeOut:
    """Minimal stand-in carrying device arrays for the selection call."""
    def __init__(self, sim, anchor, H, W):
        import paper_2605_07355_amd as ttf
        B, F, N = sim.shape
        self.B, self.F, self.H, self.W, self.C = B, F, H, W, 8
        self.buffers = ttf.TTFBuffers.allocate(B, F, H, W, 8, torch.float32, "cuda")
        self.buffers.best_sim.copy_(torch.from_numpy(sim).cuda())
        self.buffers.anchor_index.copy_(torch.from_numpy(anchor).cuda())


@pytest.mark.parametrize("fraction", [0.0, 0.05, 0.5, 0.67, 0.95, 1.0])
@pytest.mark.parametrize("B,F,H,W,ties", [(3, 5, 7, 9, False), (2, 9, 16, 16, True), (1, 2, 1, 1, False),
                                           (16, 32, 16, 16, False)])
def test_selected_threshold_is_exact(B, F, H, W, ties, fraction):
    import paper_2605_07355_amd as ttf
    from oracle import adaptive as A
    sim, anchor = similarity_field(B, F, H * W, seed=B * 100 + F, ties=ties)
    out = _FakeOut(sim, anchor, H, W)
    t = ttf.ttf_select_threshold(out, fraction)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(t.cpu().numpy(), A.select_threshold(sim, anchor, fraction))


def test_selected_threshold_without_source_frames():
    import paper_2605_07355_amd as ttf
    sim, anchor = similarity_field(4, 1, 12, seed=3)
    t = ttf.ttf_select_threshold(_FakeOut(sim, anchor, 3, 4), 0.5)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(t.cpu().numpy(), np.ones(4, np.float32))


@pytest.mark.parametrize("B,F,H,W", [(3, 5, 7, 9), (2, 1, 4, 6), (4, 12, 16, 16)])
@pytest.mark.parametrize("fraction", [0.0, 0.3, 0.67, 1.0])
def test_selected_threshold_on_segment_outputs(B, F, H, W, fraction):
    """anchor_index = -1 (outputs of ttf_compress_segment): every frame is a source frame, M = F*N,
    also for a one-frame segment."""
    import paper_2605_07355_amd as ttf
    from oracle import adaptive as A
    sim, _ = similarity_field(B, F, H * W, seed=B * 10 + F)
    anchor = np.full(B, -1, np.int32)
    t = ttf.ttf_select_threshold(_FakeOut(sim, anchor, H, W), fraction)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(t.cpu().numpy(), A.select_threshold(sim, anchor, fraction))


def test_segment_select_and_regate():
    """Threshold selection and re-gating on a segment's outputs: the threshold is the oracle's order
    statistic of the library's own similarities over all F*N tokens, and the re-gated segment fuses
    exactly the tokens above it."""
    import paper_2605_07355_amd as ttf
    from oracle import adaptive as A
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=2, F=6, C=256)
    batch = make_clip_batch(cfg)
    anchor, seg = np.ascontiguousarray(batch.x[:, 0]), np.ascontiguousarray(batch.x[:, 1:])
    out = _run_segment(seg, anchor, 3, cfg.r, cfg.t[0])
    phi = 0.5
    t = ttf.ttf_select_threshold(out, phi)
    torch.cuda.synchronize()
    sim = out.buffers.best_sim.cpu().numpy()
    np.testing.assert_array_equal(t.cpu().numpy(), A.select_threshold(sim, np.full(cfg.B, -1, np.int32), phi))
    ttf.ttf_regate(to_device(seg), out, t)
    torch.cuda.synchronize()
    M = (cfg.F - 1) * cfg.N                                        # the segment has F-1 frames, all sources
    for b in range(cfg.B):
        fused = out.buffers.fuse_map[b] >= 0
        assert torch.equal(fused, out.buffers.best_sim[b] > t[b])
        n = int(fused.sum())
        assert int(0.49 * M) <= n <= int(np.floor(float(np.float32(phi)) * M))
        assert int(out.buffers.kept_count[b]) == M - n
    assert (out.buffers.anchor_index == -1).all()


@pytest.mark.parametrize("name,scale", SMALL + [("qwen3vl_8b_batched", {})])
def test_regate_per_clip_thresholds(name, scale):
    """Search once at the workload's threshold, then re-gate at a different threshold per clip:
    every output must equal the oracle run clip by clip at those thresholds."""
    import paper_2605_07355_amd as ttf
    from oracle import adaptive as A
    cfg = CONFIGS[name].scaled(**scale)
    ts = [float(np.float32(0.45 + 0.5 * (b % 4) / 4)) for b in range(cfg.B)]     # 0.45, 0.575, 0.70, 0.825
    batch, res = _prepared(cfg, (cfg.t[0],) + tuple(sorted(set(ts) - {cfg.t[0]})))
    x, out = run_gpu(batch.x, cfg.r, cfg.t[0])
    compare_with_oracle(batch.x, out, res)
    buf = out.buffers
    buf.tokens_out.view(torch.uint8).fill_(0x7A)
    for tns in (buf.pos_ids, buf.src_index, buf.row_offsets, buf.kept_count, buf.fuse_map):
        tns.fill_(SENTINEL)
    buf.workspace.fill_(0xEE)
    ttf.ttf_regate(x, out, torch.tensor(ts, dtype=torch.float32, device="cuda"))
    torch.cuda.synchronize()
    want = A.compress_per_clip(batch.x, cfg.r, ts, res.anchor_index)
    compare_with_oracle(batch.x, out, want)
    if cfg.B > 1:
        assert len(set(want.kept_count.tolist())) > 1                 # the thresholds really differ in effect


def test_regate_with_one_threshold_equals_a_fresh_pass():
    import paper_2605_07355_amd as ttf
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=2, F=5)
    batch, res = _prepared(cfg, (0.6, 0.8))
    x, out = run_gpu(batch.x, cfg.r, 0.6)
    ttf.ttf_regate(x, out, None, t=0.8)
    torch.cuda.synchronize()
    from oracle import ttf_oracle as T
    compare_with_oracle(batch.x, out, T.compress(batch.x, cfg.r, 0.8))


def test_adaptive_end_to_end():
    """Selection on the library's own float32 similarities: the threshold is within the similarity
    tolerance of the oracle's (an order statistic moves by at most the largest perturbation), and
    the re-gated pass fuses exactly the tokens above it, at most the requested share."""
    import paper_2605_07355_amd as ttf
    from oracle import adaptive as A
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=3, F=8)
    batch = make_clip_batch(cfg)
    from oracle import ttf_oracle as T
    res = T.compress(batch.x, cfg.r, cfg.t[0], want_tokens=False)
    x, out = run_gpu(batch.x, cfg.r, cfg.t[0])
    phi = 0.4
    t = ttf.ttf_select_threshold(out, phi)
    ttf.ttf_regate(x, out, t)
    torch.cuda.synchronize()
    t_ref = A.select_threshold(res.best_sim, res.anchor_index, phi)
    assert np.abs(t.cpu().numpy().astype(np.float64) - t_ref).max() <= 1e-5
    M = (cfg.F - 1) * cfg.H * cfg.W
    sim = out.buffers.best_sim
    for b in range(cfg.B):
        src = torch.ones(cfg.F, dtype=torch.bool, device="cuda")
        src[int(out.buffers.anchor_index[b])] = False
        fused = (out.buffers.fuse_map[b] >= 0)
        assert torch.equal(fused[src], sim[b][src] > t[b])
        assert not fused[~src].any()
        n = int(fused.sum())
        assert n <= int(np.floor(float(np.float32(phi)) * M)) and n >= int(0.39 * M)
        assert int(out.buffers.kept_count[b]) == cfg.H * cfg.W + M - n


def test_new_entry_points_reject_bad_arguments():
    import paper_2605_07355_amd as ttf
    from paper_2605_07355_amd import binding as bd
    lib = ttf.load_library()
    p = bd._make_params(1, 2, 2, 2, 8, bd.TTF_F32, 1, 0.7, "auto")
    buf = torch.zeros(64, dtype=torch.int32, device="cuda")
    q = buf.data_ptr()
    assert lib.ttf_restore_map(ctypes.byref(p), None, q, q, q, None) == bd.TTF_ERR_INVALID_ARG
    assert lib.ttf_restore(ctypes.byref(p), q, -1, q, q, None) == bd.TTF_ERR_INVALID_ARG
    assert lib.ttf_restore(ctypes.byref(p), q + 4, 1, q, q, None) == bd.TTF_ERR_UNSUPPORTED
    assert lib.ttf_select_threshold(ctypes.byref(p), q, q, ctypes.c_float(1.5), q, None) == bd.TTF_ERR_INVALID_ARG
    assert lib.ttf_select_threshold(ctypes.byref(p), q, q, ctypes.c_float(float("nan")), q, None) == bd.TTF_ERR_INVALID_ARG
    o = bd._Outputs(q, q, q, q, q, q, q, None, q, None)                # best_sim missing
    assert lib.ttf_regate(ctypes.byref(p), q, None, q, 1 << 20, ctypes.byref(o), None) == bd.TTF_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert int(buf.abs().sum()) == 0


# ------------------------------------------------------------------------ streaming segments
def _segment_case(cfg, t, anchor_override=None):
    """A clip of cfg.F frames whose frame 0 plays the external anchor (or is replaced by
    `anchor_override` [B,H,W,C]); margins enforced against that anchor."""
    from oracle import margins
    for attempt in range(4):
        batch = make_clip_batch(cfg, seed=cfg.seed + 1000 * attempt)
        if anchor_override is not None:
            batch.x[:, 0] = anchor_override
        try:
            margins.enforce_margins(batch, cfg.r, (t,), ANCHOR_FIXED, 0, want_tokens=False)
            return batch
        except margins.MarginError:
            continue
    raise RuntimeError("no seed met the margins")


def _run_segment(seg_np, anchor_np, frame_offset, r, t):
    import paper_2605_07355_amd as ttf
    x, a = to_device(np.ascontiguousarray(seg_np)), to_device(np.ascontiguousarray(anchor_np))
    B, F, H, W, C = x.shape
    buf = ttf.TTFBuffers.allocate(B, F, H, W, C, x.dtype, x.device)
    buf.tokens_out.view(torch.uint8).fill_(0x7A)
    for tns in (buf.pos_ids, buf.src_index, buf.row_offsets, buf.kept_count, buf.anchor_index, buf.fuse_map,
                buf.best_idx):
        tns.fill_(SENTINEL)
    buf.best_sim.fill_(float("nan"))
    buf.workspace.fill_(0xCD)
    out = ttf.ttf_compress_segment(x, a, frame_offset, r=r, t=t, buffers=buf)
    torch.cuda.synchronize()
    return out


def _compare_segment(seg_np, out, want):
    """Segment outputs against the oracle's SegmentResult (same bar as the whole pass)."""
    from types import SimpleNamespace
    B = seg_np.shape[0]
    shim = SimpleNamespace(anchor_index=np.full(B, -1, np.int32), fuse_map=want.fuse_map, kept_count=want.kept_count,
                           row_offsets=want.row_offsets, src_index=want.src_index, pos_ids=want.pos_ids,
                           best_idx=want.best_idx, best_sim=want.best_sim, total_rows=want.total_rows)
    compare_with_oracle(seg_np, out, shim)


SEGMENTS = [
    ("tiny", {}, 1),
    ("qwen3vl_2b", dict(B=2, F=6), 1),                                 # matrix-core path, 5 source frames
    ("qwen3vl_2b", dict(B=1, F=2), 1),                                 # one-frame segment
    ("qwen3vl_2b", dict(B=2, F=10, C=256), 2),                         # more frames than one workgroup group
    ("highres_wide", dict(B=1, F=4, H=8, C=128), 2),                   # 32-wide grid
    ("highres_wide", dict(B=2, F=18, H=64, C=128), 2),                 # LDS-shared anchor kernel, 17 source frames
    ("tiny", dict(B=3, F=5, H=7, W=9, C=40, dtype="f32"), 1),          # general kernels, ragged keep words
    ("tiny", dict(B=2, F=3, H=5, W=13, C=129, dtype="bf16"), 3),
    ("qwen3vl_2b", dict(B=2, F=7, H=14, W=14, C=128), 1),              # padded tile rows, external anchor
    ("qwen3vl_2b", dict(B=1, F=4, H=9, W=24, C=256), 2),
    ("qwen3vl_2b", dict(B=1, F=6, H=7, W=44, C=128), 1),               # wider than 32
    ("tiny", dict(B=2, F=4, H=5, W=7, C=1540, dtype="f32"), 1),        # long rows: one block per token
    ("qwen3vl_2b", dict(B=6, F=6, C=128, dtype="f32"), 1),             # fp32 on the matrix cores, external anchor
    ("qwen3vl_2b", dict(B=7, F=5, H=14, W=14, C=64, dtype="f32"), 2),  # the same on padded tile rows, 5x5 window
]


@pytest.mark.parametrize("name,scale,r", SEGMENTS)
def test_segment_against_external_anchor(name, scale, r):
    from oracle import streaming as S
    cfg = CONFIGS[name].scaled(**{**scale, "r": r})
    t = cfg.t[0]
    batch = _segment_case(cfg, t)
    anchor, seg = batch.x[:, 0], batch.x[:, 1:]
    want = S.compress_segment(seg, anchor, r, t, frame_offset=40)
    out = _run_segment(seg, anchor, 40, r, t)
    _compare_segment(np.ascontiguousarray(seg), out, want)
    assert 0 < (want.fuse_map >= 0).mean() < 1


def test_segment_at_headline_size():
    """31 source frames per clip of the headline workload against its first frame."""
    from oracle import streaming as S
    cfg = CONFIGS["qwen3vl_8b_batched"]
    t = cfg.t[0]
    batch = _segment_case(cfg, t)
    anchor, seg = batch.x[:, 0], np.ascontiguousarray(batch.x[:, 1:])
    want = S.compress_segment(seg, anchor, cfg.r, t, frame_offset=1)
    out = _run_segment(seg, anchor, 1, cfg.r, t)
    _compare_segment(seg, out, want)


def test_rolling_anchor_chain():
    """Two segments of one stream: the second is matched against the last frame of the first, and
    the appended rows carry stream-wide frame numbers."""
    from oracle import streaming as S
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=2, F=5, C=512)
    t = cfg.t[0]
    first = _segment_case(cfg, t)
    second = _segment_case(cfg, t, anchor_override=first.x[:, -1])
    stream_rows = 0
    anchor = first.x[:, 0]
    for n, batch in enumerate((first, second)):
        seg = np.ascontiguousarray(batch.x[:, 1:])
        off = 1 + n * (cfg.F - 1)
        want = S.compress_segment(seg, anchor, cfg.r, t, frame_offset=off)
        out = _run_segment(seg, anchor, off, cfg.r, t)
        _compare_segment(seg, out, want)
        pos = out.buffers.pos_ids[0, :want.total_rows]
        assert int(pos.min()) >= off and int(pos.max()) < off + cfg.F - 1
        stream_rows += want.total_rows
        anchor = seg[:, -1]                                            # rolling anchor for the next segment
    assert 0 < stream_rows < 2 * cfg.B * (cfg.F - 1) * cfg.H * cfg.W


@pytest.mark.parametrize("C", [256, 1024])             # short rows, and long rows (copy driven by a row count of 0)
def test_static_stream_appends_nothing(C):
    import paper_2605_07355_amd as ttf
    from workloads.ttf_gen import identical_frames, f32_to_bf16_bits
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=2, F=4, C=C)
    x = f32_to_bf16_bits(identical_frames(cfg, seed=5))
    out = _run_segment(x[:, 1:], x[:, 0], 1, 1, 0.9)
    assert out.total_rows == 0
    np.testing.assert_array_equal(out.buffers.kept_count.cpu().numpy(), [0, 0])
    np.testing.assert_array_equal(out.buffers.anchor_index.cpu().numpy(), [-1, -1])
    fm = out.buffers.fuse_map.cpu().numpy()
    np.testing.assert_array_equal(fm, np.broadcast_to(np.arange(cfg.H * cfg.W), fm.shape))


def test_segment_rejects_bad_arguments():
    import paper_2605_07355_amd as ttf
    from paper_2605_07355_amd import binding as bd
    lib = ttf.load_library()
    p = bd._make_params(1, 2, 2, 2, 8, bd.TTF_F32, 1, 0.7, "auto")
    buf = torch.zeros(4096, dtype=torch.int32, device="cuda")
    q = buf.data_ptr()
    o = bd._Outputs(q, q, q, q, q, q, q, None, None, None)
    assert lib.ttf_compress_segment(ctypes.byref(p), q, None, 0, q, 1 << 20, ctypes.byref(o), None) == bd.TTF_ERR_INVALID_ARG
    assert lib.ttf_compress_segment(ctypes.byref(p), q, q + 4, 0, q, 1 << 20, ctypes.byref(o), None) == bd.TTF_ERR_UNSUPPORTED
    assert lib.ttf_compress_segment(ctypes.byref(p), q, q, 2 ** 31 - 2, q, 1 << 20, ctypes.byref(o), None) == bd.TTF_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert int(buf.abs().sum()) == 0


# ------------------------------------------------------------------------------ tied batch
def _tied_case(cfg, t, anchor="auto"):
    from oracle import margins
    mode, idx = (ANCHOR_AUTO, 0) if anchor == "auto" else (ANCHOR_FIXED, int(anchor))
    for attempt in range(4):
        batch = make_clip_batch(cfg, seed=cfg.seed + 1000 * attempt)
        try:
            return batch, margins.enforce_tied_margins(batch, cfg.r, (t,), mode, idx, want_tokens=True)
        except margins.MarginError:
            continue
    raise RuntimeError("no seed met the margins")


def _run_tied(x_np, r, t, anchor="auto"):
    import paper_2605_07355_amd as ttf
    x = to_device(x_np)
    B, F, H, W, C = x.shape
    buf = ttf.TTFTiedBuffers.allocate(B, F, H, W, C, x.dtype, x.device, r=r)
    buf.tokens_out.view(torch.uint8).fill_(0x7A)
    for tns in (buf.pos_ids, buf.src_index, buf.kept_count, buf.anchor_index, buf.fuse_map, buf.best_idx):
        tns.fill_(SENTINEL)
    buf.best_sim.fill_(float("nan"))
    buf.mean_sim.fill_(float("nan"))
    buf.workspace.fill_(0xCD)
    ttf.ttf_compress_tied(x, r=r, t=t, anchor=anchor, buffers=buf)
    torch.cuda.synchronize()
    return buf


def _compare_tied(x_np, buf, res):
    B, F, H, W, C = x_np.shape
    N = H * W
    n = res.kept_count
    np.testing.assert_array_equal(buf.anchor_index.cpu().numpy(), np.full(B, res.anchor_index))
    np.testing.assert_array_equal(buf.best_idx.cpu().numpy(), res.best_idx)
    np.testing.assert_array_equal(buf.fuse_map.cpu().numpy(), res.fuse_map)
    assert int(buf.kept_count[0]) == n
    src = buf.src_index.cpu().numpy()
    np.testing.assert_array_equal(src[:n], res.src_index[:n])
    assert (src[n:] == SENTINEL).all()
    pos = buf.pos_ids.cpu().numpy()
    np.testing.assert_array_equal(pos[:, :n], res.pos_ids[:, :n])
    assert (pos[:, n:] == SENTINEL).all()
    assert np.abs(buf.best_sim.cpu().numpy().astype(np.float64) - res.best_sim).max() <= 1e-5
    assert np.abs(buf.mean_sim.cpu().numpy().astype(np.float64) - res.mean_sim).max() <= 1e-5
    bits = np.uint16 if x_np.dtype == np.uint16 else np.uint32
    got = rows_as_bits(buf.tokens_out.view(B * F * N, C)).reshape(B, F * N, C)
    xin = x_np.reshape(B, F * N, C).view(bits)
    fill = 0x7A7A if bits == np.uint16 else 0x7A7A7A7A
    for b in range(B):
        np.testing.assert_array_equal(got[b, :n], xin[b][res.src_index[:n]])
        assert (got[b, n:] == fill).all()


TIED = [
    ("qwen3vl_2b", dict(B=3, F=6), 1, "auto"),                              # matrix-core path
    ("qwen3vl_2b", dict(B=2, F=4, C=256), 2, "auto"),
    ("qwen3vl_2b", dict(B=4, F=5, C=128), 0, 2),
    ("highres_wide", dict(B=2, F=4, H=8, C=128), 2, "auto"),                # 32-wide grid
    ("highres_wide", dict(B=2, F=3, H=4, C=128), 1, -1),
    ("tiny", dict(B=3, F=5, H=7, W=9, C=40, dtype="f32"), 1, "auto"),       # general kernels
    ("qwen3vl_2b", dict(B=6, F=5, C=128, dtype="f32"), 1, "auto"),          # fp32 on the matrix cores
    ("qwen3vl_2b", dict(B=6, F=4, H=9, W=24, C=64, dtype="f32"), 2, "auto"),   # fp32, padded tile rows
    ("tiny", dict(B=2, F=4, H=5, W=13, C=129, dtype="bf16"), 3, "auto"),
    ("tiny", dict(B=1, F=4, H=6, W=6, C=64, dtype="bf16"), 1, "auto"),      # B = 1: the plain pass
    ("qwen3vl_2b", dict(B=2, F=1, C=128), 1, "auto"),                       # no source frame
    ("qwen3vl_2b", dict(B=2, F=5, C=96), 1, "auto"),                        # 3 K-steps over four waves
    ("qwen3vl_2b", dict(B=2, F=4, H=10, W=20, C=160), 2, "auto"),           # padded tile rows, 5 K-steps
    ("qwen3vl_2b", dict(B=3, F=4, H=14, W=14, C=128), 1, "auto"),           # 14x14: padded tile rows
    ("qwen3vl_2b", dict(B=2, F=5, H=9, W=24, C=256), 2, "auto"),
    ("qwen3vl_2b", dict(B=2, F=6, H=5, W=44, C=128), 1, 0),                 # wider than 32
    ("qwen3vl_2b", dict(B=3, F=3, H=7, W=16, C=128), 0, "auto"),            # 16 wide, partial keep words
    ("tiny", dict(B=3, F=24, H=64, W=16, C=40, dtype="f32"), 1, "auto"),    # large general input: LDS-tiled kernel
    ("highres_wide", dict(B=2, F=18, H=64, C=128), 2, "auto"),              # LDS-shared anchor kernel, all-window form
    ("tiny", dict(B=3, F=4, H=5, W=7, C=1540, dtype="f32"), 1, "auto"),     # long rows: one block per token
]


@pytest.mark.parametrize("name,scale,r,anchor", TIED)
def test_tied_batch(name, scale, r, anchor):
    cfg = CONFIGS[name].scaled(**{**scale, "r": r, "shared_motion": True})
    t = cfg.t[0]
    batch, res = _tied_case(cfg, t, anchor)
    buf = _run_tied(batch.x, r, t, anchor)
    _compare_tied(batch.x, buf, res)
    if cfg.F > 1 and cfg.B > 1:
        assert 0 < (res.fuse_map >= 0).mean() < 1


def test_tied_batch_at_headline_size():
    cfg = CONFIGS["qwen3vl_8b_batched"].scaled(shared_motion=True)
    t = cfg.t[0]
    batch, res = _tied_case(cfg, t)
    buf = _run_tied(batch.x, cfg.r, t)
    _compare_tied(batch.x, buf, res)
    assert (res.fuse_map >= 0).mean() > 0.2


def test_tied_rejects_bad_arguments():
    import paper_2605_07355_amd as ttf
    from paper_2605_07355_amd import binding as bd
    lib = ttf.load_library()
    p = bd._make_params(2, 2, 2, 2, 8, bd.TTF_F32, 4, 0.7, "auto")            # r = 4 is beyond the mode's limit
    n = ctypes.c_size_t(0)
    assert lib.ttf_tied_workspace_size(ctypes.byref(p), ctypes.byref(n)) == bd.TTF_ERR_UNSUPPORTED
    p = bd._make_params(2, 2, 2, 2, 8, bd.TTF_F32, 1, 0.7, "auto")
    buf = torch.zeros(1 << 16, dtype=torch.int32, device="cuda")
    q = buf.data_ptr()
    o = bd._TiedOutputs(q, q, q, q, q, None, None, None, None, None)         # fuse_map missing
    assert lib.ttf_compress_tied(ctypes.byref(p), q, q, 1 << 18, ctypes.byref(o), None) == bd.TTF_ERR_INVALID_ARG
    o = bd._TiedOutputs(q, q, q, q, q, q, None, None, None, None)
    assert lib.ttf_compress_tied(ctypes.byref(p), q, q, 16, ctypes.byref(o), None) == bd.TTF_ERR_WORKSPACE_TOO_SMALL
    torch.cuda.synchronize()
    assert int(buf.abs().sum()) == 0


@pytest.mark.parametrize("H,W,C,dtype", [(4, 16, 128, "bf16"), (3, 5, 24, "f32")])
def test_tied_ties_go_to_the_lowest_index(H, W, C, dtype):
    """The anchor frame repeats a token in neighbouring cells and all frames are identical: equal
    batch-mean similarities and equal anchor scores must resolve to the first maximum."""
    from oracle import ttf_oracle as T
    from workloads import f32_to_bf16_bits
    rng = np.random.default_rng(51)
    frame = rng.standard_normal((3, H, W, C)).astype(np.float32)
    frame[:, :, 2] = frame[:, :, 1]
    x = np.repeat(frame[:, None], 3, axis=1)
    x = f32_to_bf16_bits(x) if dtype == "bf16" else x
    res = T.compress_tied(x, 1, 0.5)
    assert res.anchor_index == 0 and (res.best_idx[1].reshape(H, W)[:, 2] == np.arange(H) * W + 1).all()
    buf = _run_tied(x, 1, 0.5)
    _compare_tied(x, buf, res)


def _random_segment_shapes(n, seed):
    rng = np.random.default_rng(seed)
    widths = [3, 15, 16, 17, 24, 32, 33, 47, 48, 50]
    out = []
    for _ in range(n):
        out.append((int(rng.integers(1, 4)), int(rng.integers(2, 11)), int(rng.integers(1, 11)), int(rng.choice(widths)),
                    int(rng.choice([128, 256, 96])), "bf16" if rng.random() < 0.8 else "f32", int(rng.choice([0, 1, 2, 3]))))
    return out


@pytest.mark.parametrize("B,F,H,W,C,dtype,r", _random_segment_shapes(20, seed=20260102))
def test_random_segments(B, F, H, W, C, dtype, r):
    """Seeded small segments across every search path: frame 0 of a generated clip is the external
    anchor, the rest is the segment."""
    from oracle import streaming as S
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=B, F=F, H=H, W=W, C=C, dtype=dtype, r=r, max_offset=min(max(r, 1), 2),
                                       sigma=0.5, region=2, seed=700 + B + 3 * F + 5 * H + 7 * W + C + r)
    t = cfg.t[0]
    batch = _segment_case(cfg, t)
    anchor, seg = batch.x[:, 0], np.ascontiguousarray(batch.x[:, 1:])
    want = S.compress_segment(seg, anchor, r, t, frame_offset=3)
    out = _run_segment(seg, anchor, 3, r, t)
    _compare_segment(seg, out, want)


def test_follow_on_calls_are_reproducible_and_honour_the_stream():
    """Every follow-on entry point enqueues on the stream it is given (here a side stream that
    also carries the upload) and gives bit-identical results when repeated."""
    import paper_2605_07355_amd as ttf
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=3, F=6, H=12, W=20, C=128, shared_motion=True)
    x_np = make_clip_batch(cfg).x
    side = torch.cuda.Stream()
    host = torch.from_numpy(x_np.view(np.int16)).pin_memory()
    runs = []
    for _ in range(2):
        with torch.cuda.stream(side):
            x = torch.empty(host.shape, dtype=torch.int16, device="cuda")
            x.copy_(host, non_blocking=True)                         # the calls below must wait for this copy
            x = x.view(torch.bfloat16)
            out = ttf.ttf_compress(x, r=1, t=0.7, stream=side)
            rmap = ttf.ttf_restore_map(out, stream=side)
            full = ttf.ttf_restore(out.buffers.tokens_out, cfg.tokens, rmap, cfg.H, cfg.W, stream=side)
            thr = ttf.ttf_select_threshold(out, 0.5, stream=side)
            snap = [t.clone() for t in (out.buffers.fuse_map, out.buffers.kept_count, rmap, full.view(torch.int16), thr)]
            ttf.ttf_regate(x, out, thr, stream=side)
            seg = ttf.ttf_compress_segment(x[:, 1:].contiguous(), x[:, 0].contiguous(), 1, r=1, t=0.7, stream=side)
            tied = ttf.ttf_compress_tied(x, r=1, t=0.7, stream=side)
            snap += [t.clone() for t in (out.buffers.fuse_map, out.buffers.row_offsets, seg.buffers.fuse_map,
                                         seg.buffers.row_offsets, tied.fuse_map, tied.kept_count, tied.best_sim)]
        side.synchronize()
        runs.append(snap)
    for first, second in zip(*runs):
        assert torch.equal(first, second)
    assert int(runs[0][1].sum()) > 0
