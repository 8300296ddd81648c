#!/usr/bin/env python3
"""Benchmark of the TTF pass on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]

A step is one ttf_compress call (all stages: anchor selection, window search + gate, offsets
scan, row emission) on one synthetic batch that is already resident in HBM.  Prints one JSON
line: whole-path throughput in GTok/s, the roofline of the dominant kernel from HIP events
recorded on the launch stream, and the CPU oracle timed on this machine's host cores.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published peak


def kernel_source_digest() -> str:
    """Digest of the kernel sources; counter-derived traffic figures are tied to it."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2605_07355_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        with open(os.path.join(csrc, name), "rb") as fh:
            h.update(name.encode())
            h.update(fh.read())
    return h.hexdigest()[:16]


def measured_traffic(workload: str, stage: str):
    """HBM bytes per launch of `stage` from committed rocprofv3 counter runs, or None when
    there are none for the current kernel sources."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as fh:
            rec = json.load(fh)
    except (OSError, ValueError):
        return None
    if rec.get("kernel_source_digest") != kernel_source_digest():
        return None
    return rec.get("bytes_per_launch", {}).get(workload, {}).get(stage)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="qwen3vl_8b_batched")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extensions", action="store_true",
                    help="skip the timings of restoration, adaptive threshold and streaming segments")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this benchmark runs on one GPU only; clips shard across GPUs with no communication, "
              "but no multi-GPU path is built or measured. Use --gpus 1.", file=sys.stderr)
        return 2
    if int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: WORLD_SIZE > 1 is not supported (one GPU only).", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2605_07355_amd as ttf
    from workloads import CONFIGS, make_clip_batch

    cfg = CONFIGS[args.workload]
    r, t = cfg.r, cfg.t[0]
    batch = make_clip_batch(cfg)
    dev = torch.device("cuda:0")
    if cfg.dtype == "bf16":
        x = torch.from_numpy(batch.x.view(np.int16)).to(dev).view(torch.bfloat16)
    else:
        x = torch.from_numpy(batch.x).to(dev)
    buf = ttf.TTFBuffers.allocate(cfg.B, cfg.F, cfg.H, cfg.W, cfg.C, x.dtype, dev, want_sim=True)
    stream = torch.cuda.current_stream(dev)
    steps, warmup = max(1, args.steps), max(0, args.warmup)

    def step():
        ttf.ttf_compress(x, r=r, t=t, anchor="auto", buffers=buf, stream=stream)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / steps
    tokens = cfg.tokens
    gtok_s = tokens / (elapsed / steps) / 1e9

    # Same loop again with HIP events recorded around every stage on the launch stream.
    slots = min(steps, 256)
    ttf.ttf_profile_enable(slots)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(slots):
        step()
    torch.cuda.synchronize()
    prof_elapsed = time.perf_counter() - t1
    stage_ms = {n: 0.0 for n in ttf.STAGE_NAMES}
    for c in range(slots):
        for n, v in ttf.ttf_profile_read(c).items():
            stage_ms[n] += v / slots
    ttf.ttf_profile_enable(0)

    # Practical ceiling: a plain device-to-device copy of the input (reads + writes counted).
    scratch = torch.empty_like(x)
    for _ in range(2):
        scratch.copy_(x)
    torch.cuda.synchronize()
    c0 = time.perf_counter()
    for _ in range(5):
        scratch.copy_(x)
    torch.cuda.synchronize()
    copy_gbps = 5 * 2 * x.numel() * x.element_size() / (time.perf_counter() - c0) / 1e9
    del scratch

    kept = buf.kept_count.cpu().numpy().astype(np.int64)
    rows = int(kept.sum())
    kappa = rows / tokens
    fused_fraction = float((buf.fuse_map >= 0).sum().item()) / max(1, cfg.B * (cfg.F - 1) * cfg.N)
    row_bytes = cfg.C * cfg.elem_bytes

    # Algorithmic bytes per launch (per input token x tokens per launch):
    #   frame sums:     C*e                       every row read once for the anchor rule
    #   window search:  C*e + 12                  every row read once (source rows and, once per clip,
    #                                             the anchor frame) + best_sim, best_idx, fuse_map
    #   emit rows:      kappa * (2*C*e + 16)      kept rows read and written + position ids, src_index
    #   anchor norms:   C*e / F                   the anchor frame once more for its norms
    # whole path: (2 + 1/F + kappa) * C*e per token -- kept rows are counted once (their write); the
    # re-read of kept rows by the emit kernel is an implementation cost, not algorithmic.
    alg_bytes = {
        "frame_sums": tokens * row_bytes,
        "window_search": tokens * (row_bytes + 12),
        "emit_rows": rows * (2 * row_bytes + 16),
        "anchor_norms": tokens * row_bytes // cfg.F,
    }
    path_bytes = (2.0 + 1.0 / cfg.F + kappa) * row_bytes * tokens
    dominant = max(alg_bytes, key=lambda n: stage_ms.get(n, 0.0))
    dom_ms = stage_ms[dominant]
    achieved = alg_bytes[dominant] / (dom_ms * 1e-3) / 1e9 if dom_ms > 0 else 0.0
    roofline = {
        "kernel": dominant, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
        "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
        "avg_kernel_ms": round(dom_ms, 4),
        "algorithmic_bytes_per_launch": int(alg_bytes[dominant]),
        "traffic": measured_traffic(cfg.name, dominant),
    }
    path = {
        "algorithmic_bytes_per_step": int(path_bytes),
        "achieved_GBps": round(path_bytes / (elapsed / steps) / 1e9, 1),
        "frac_of_hbm_peak": round(path_bytes / (elapsed / steps) / 1e9 / HBM_PEAK_GBPS, 4),
        "stage_ms": {n: round(v, 4) for n, v in stage_ms.items()},
        "stage_GBps": {n: round(alg_bytes[n] / (stage_ms[n] * 1e-3) / 1e9, 1)
                       for n in alg_bytes if stage_ms.get(n, 0) > 0},
        "ms_per_step_with_stage_events": round(1e3 * prof_elapsed / slots, 4),
        "device_copy_GBps": round(copy_gbps, 1),
        "kappa": round(kappa, 4), "fused_fraction": round(fused_fraction, 4),
        "reduction_ratio": round(1.0 - kappa, 4),
    }

    # The entry points built on top of the pass, timed with events on the same stream.  Each
    # figure is the mean of `reps` back-to-back calls; GB/s counts algorithmic bytes only.
    extensions = None
    if not args.no_extensions:
        reps = 10

        def timed(fn):
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(reps):
                fn()
            e1.record(stream)
            e1.synchronize()
            return e0.elapsed_time(e1) / reps

        def entry(ms, nbytes, **kw):
            return {"ms": round(ms, 4), "algorithmic_bytes": int(nbytes),
                    "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
                    "frac_of_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4), **kw}

        out = ttf.TTFOutput(buf, cfg.B, cfg.F, cfg.H, cfg.W, cfg.C)
        rmap = torch.empty((cfg.B, cfg.F, cfg.N), dtype=torch.int32, device=dev)
        full = torch.empty_like(x)
        extensions = {}
        ms = timed(lambda: ttf.ttf_restore_map(out, rmap))
        extensions["restore_map"] = entry(ms, 8 * tokens + 4 * rows)            # fuse_map in, map out, src_index in
        ms = timed(lambda: ttf.ttf_restore(buf.tokens_out, rows, rmap, cfg.H, cfg.W, full))
        extensions["restore"] = entry(ms, (tokens + rows) * row_bytes + 4 * tokens)   # unique rows in, full layout out
        del full
        thr = torch.empty((cfg.B,), dtype=torch.float32, device=dev)
        ms = timed(lambda: ttf.ttf_select_threshold(out, 0.67, thr))
        extensions["select_threshold"] = entry(ms, 4 * tokens, fused_fraction_requested=0.67)
        ms = timed(lambda: ttf.ttf_regate(x, out, thr))
        rows_rg = int(buf.kept_count.sum().item())
        extensions["regate"] = entry(ms, 12 * tokens + rows_rg * (2 * row_bytes + 16), rows=rows_rg)
        # fixed anchor (the paper's first / last frame ablation): no pass for the anchor rule
        ms = timed(lambda: ttf.ttf_compress(x, r=r, t=t, anchor=0, buffers=buf, stream=stream))
        rows_fx = int(buf.kept_count.sum().item())
        extensions["compress_fixed_anchor"] = entry(
            ms, (1.0 + 1.0 / cfg.F) * row_bytes * tokens + rows_fx * row_bytes, anchor="first frame", rows=rows_fx,
            GTok_per_s=round(tokens / (ms * 1e-3) / 1e9, 4))
        # one stream segment: frames 1..F-1 of every clip against frame 0 as the rolling anchor
        if cfg.F > 1:
            seg = x[:, 1:].contiguous()
            anc = x[:, 0].contiguous()
            sbuf = ttf.TTFBuffers.allocate(cfg.B, cfg.F - 1, cfg.H, cfg.W, cfg.C, x.dtype, dev, want_sim=True)
            ms = timed(lambda: ttf.ttf_compress_segment(seg, anc, 1, r=r, t=t, buffers=sbuf))
            seg_tokens = cfg.B * (cfg.F - 1) * cfg.N
            seg_rows = int(sbuf.kept_count.sum().item())
            nbytes = seg_tokens * (row_bytes + 12) + cfg.B * cfg.N * row_bytes + seg_rows * (2 * row_bytes + 16)
            extensions["compress_segment"] = entry(ms, nbytes, source_tokens=seg_tokens, rows=seg_rows,
                                                   GTok_per_s=round(seg_tokens / (ms * 1e-3) / 1e9, 4))
            del seg, anc, sbuf
        # tied-batch mode on a batch whose clips share their motion (views of one scene dynamics)
        if cfg.r <= 3:
            tb = make_clip_batch(cfg.scaled(shared_motion=True))
            if cfg.dtype == "bf16":
                xt = torch.from_numpy(tb.x.view(np.int16)).to(dev).view(torch.bfloat16)
            else:
                xt = torch.from_numpy(tb.x).to(dev)
            del tb
            tbuf = ttf.TTFTiedBuffers.allocate(cfg.B, cfg.F, cfg.H, cfg.W, cfg.C, xt.dtype, dev, r=r)
            ms = timed(lambda: ttf.ttf_compress_tied(xt, r=r, t=t, buffers=tbuf))
            lp = int(tbuf.kept_count.item())
            kwin = (2 * r + 1) ** 2
            # both passes over the input, the window similarities written and read once, shared
            # outputs, and the kept rows of every element written
            nbytes = ((2.0 + 1.0 / cfg.F) * row_bytes + 8 * kwin + 4) * tokens + cfg.B * lp * row_bytes
            extensions["compress_tied"] = entry(ms, nbytes, rows_per_element=lp,
                                                fused_fraction=round(float((tbuf.fuse_map >= 0).sum().item())
                                                                     / max(1, (cfg.F - 1) * cfg.N), 4),
                                                GTok_per_s=round(tokens / (ms * 1e-3) / 1e9, 4))
            del xt, tbuf
        ttf.ttf_compress(x, r=r, t=t, anchor="auto", buffers=buf, stream=stream)   # leave buf as the pass wrote it
        torch.cuda.synchronize()

    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import ttf_oracle as orc
        orc.build(force=False)
        c0 = time.perf_counter()
        ref = orc.compress(batch.x, r, t, want_tokens=True)
        cpu_s = time.perf_counter() - c0
        agree = bool(np.array_equal(ref.kept_count, kept)) and \
            bool(np.array_equal(ref.anchor_index, buf.anchor_index.cpu().numpy()))
        cpu_baseline = {
            "value": round(tokens / cpu_s / 1e9, 6), "unit": "GTok/s", "cores": orc.threads(),
            "kind": "oracle", "seconds": round(cpu_s, 3),
            "sample": f"the whole {cfg.name} batch ({tokens} tokens), one run of the fp64 oracle",
            "counts_agree_with_gpu": agree,
        }

    line = {
        "metric": "ttf_visual_tokens_per_sec", "value": round(gtok_s, 5), "unit": "GTok/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "B": cfg.B, "F": cfg.F, "H": cfg.H, "W": cfg.W, "C": cfg.C,
                   "r": r, "t": t, "anchor": "auto", "tokens": tokens, "input_bytes": tokens * row_bytes,
                   "inputs": "resident in HBM before the timed region"
                             + ("; the same tensor every step and small enough for the 256 MiB Infinity Cache "
                                "(cache-resident run: no bandwidth claim)" if tokens * row_bytes <= (192 << 20) else "")},
        "roofline": roofline, "path": path, "cpu_baseline": cpu_baseline, "extensions": extensions,
        "context": "paper reports ~67% of tokens removed at t=0.70 and ~0.16 GFLOPs matching cost on an "
                   "A100 40GB; no timing of the pass itself",
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
