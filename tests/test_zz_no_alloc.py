"""GPU test of ttf_compress_static, the entry point that allocates nothing: its workspace is an
array inside the library's device image.  Its outputs must equal ttf_compress's (same kernels, so
bit for bit) on two calls in a row, the second on a smaller input, and sizes beyond the built-in
workspace must be refused before anything is launched."""
import ctypes

import numpy as np
import pytest
import torch

from workloads import CONFIGS, make_clip_batch

from helpers import SENTINEL, to_device

pytestmark = pytest.mark.gpu

FIELDS = ("tokens_out", "pos_ids", "src_index", "row_offsets", "kept_count", "anchor_index", "fuse_map",
          "best_sim", "best_idx")


def _poisoned(ttf, x):
    B, F, H, W, C = x.shape
    buf = ttf.TTFBuffers.allocate(B, F, H, W, C, x.dtype, x.device, want_sim=True)
    buf.tokens_out.view(torch.uint8).fill_(0x7A)
    for name in ("pos_ids", "src_index", "row_offsets", "kept_count", "anchor_index", "fuse_map", "best_idx"):
        getattr(buf, name).fill_(SENTINEL)
    buf.best_sim.fill_(float("nan"))
    return buf


def _same_as_workspace_call(ttf, cfg, seed):
    x = to_device(make_clip_batch(cfg, seed=seed).x)
    got, ref = _poisoned(ttf, x), _poisoned(ttf, x)
    ref.workspace.fill_(0xCD)
    ttf.ttf_compress(x, r=cfg.r, t=cfg.t[0], buffers=ref)
    got.workspace = None                                         # the static call must not need one
    ttf.ttf_compress_static(x, got, r=cfg.r, t=cfg.t[0])
    torch.cuda.synchronize()
    assert int(ref.row_offsets[-1]) > cfg.B * cfg.N              # some source rows survive
    for name in FIELDS:
        a, b = getattr(got, name), getattr(ref, name)
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), name   # untouched tails included
    return x


def test_static_workspace_matches_caller_workspace_twice():
    import paper_2605_07355_amd as ttf
    big = CONFIGS["qwen3vl_2b"].scaled(B=2, F=8, C=512)                       # matrix-core path
    small = CONFIGS["tiny"].scaled(B=1, F=4, H=7, W=9, C=40)                 # fp32, general path, ragged
    assert ttf.ttf_workspace_size(big.B, big.F, big.H, big.W, big.C, torch.bfloat16) <= ttf.TTF_STATIC_WORKSPACE_BYTES
    _same_as_workspace_call(ttf, big, seed=31)
    _same_as_workspace_call(ttf, small, seed=32)                             # the array still holds the first call's data
    _same_as_workspace_call(ttf, big, seed=33)


def test_static_workspace_refuses_large_problems():
    import paper_2605_07355_amd as ttf
    from paper_2605_07355_amd import binding
    cfg = CONFIGS["qwen3vl_8b_batched"]
    assert ttf.ttf_workspace_size(cfg.B, cfg.F, cfg.H, cfg.W, cfg.C, torch.bfloat16) > ttf.TTF_STATIC_WORKSPACE_BYTES
    lib = ttf.load_library()
    p = binding._Params(cfg.B, cfg.F, cfg.H, cfg.W, cfg.C, binding.TTF_BF16, 1, 0.7, 0, 0)
    canary = torch.full((64,), SENTINEL, dtype=torch.int32, device="cuda")
    o = binding._Outputs(*([canary.data_ptr()] * 9), None)
    st = lib.ttf_compress_static(ctypes.byref(p), canary.data_ptr(), ctypes.byref(o), None)
    assert st == binding.TTF_ERR_WORKSPACE_TOO_SMALL
    torch.cuda.synchronize()
    assert (canary == SENTINEL).all()                            # nothing was launched
    assert lib.ttf_compress_static(ctypes.byref(p), None, ctypes.byref(o), None) == binding.TTF_ERR_INVALID_ARG
