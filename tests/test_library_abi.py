"""CPU-only checks of the boundary: the shared library loads, exports every symbol the header
declares, sizes its workspace, and rejects bad arguments before touching the GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "ttf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ttf_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    import paper_2605_07355_amd as ttf
    lib = ttf.load_library()
    names = _declared_symbols()
    assert {"ttf_compress", "ttf_workspace_size", "ttf_status_string", "ttf_last_hip_error"} <= set(names)
    for n in names:
        assert getattr(lib, n) is not None, n


def test_status_strings():
    import paper_2605_07355_amd as ttf
    seen = {ttf.ttf_status_string(i) for i in range(5)}
    assert len(seen) == 5 and "ok" in seen
    assert ttf.ttf_status_string(99) == "unknown status"
    assert ttf.ttf_last_hip_error() == 0
    assert len(ttf.STAGE_NAMES) == 7 and all(ttf.STAGE_NAMES)


def test_workspace_size_and_argument_checks():
    import torch
    import paper_2605_07355_amd as ttf
    n = ttf.ttf_workspace_size(16, 32, 16, 16, 4096, torch.bfloat16)
    # frame sums [B,F,C] fp32 (8 MiB) + the anchor frames in fragment order [B,N,C] bf16 (32 MiB)
    # + the 32-token strip sums of the speculative anchor route [B,F,N/32,C] fp32 (64 MiB)
    # + small per-token / per-frame arrays
    assert 104 * 2**20 <= n <= 107 * 2**20
    # no strip sums where that route does not exist (here: fewer than 1024 channels)
    assert ttf.ttf_workspace_size(16, 32, 16, 16, 512, torch.bfloat16) <= 6 * 2**20
    # fp32 with whole 32-channel K-steps: the anchor frames as three bf16 planes (48 MiB here)
    assert 52 * 2**20 <= ttf.ttf_workspace_size(16, 32, 16, 16, 2048, torch.float32) <= 53 * 2**20
    assert ttf.ttf_workspace_size(16, 32, 16, 16, 2040, torch.float32) <= 5 * 2**20
    assert ttf.ttf_workspace_size(1, 1, 1, 1, 1, torch.float32) > 0
    for bad in (dict(B=0), dict(F=0), dict(H=-1), dict(C=0), dict(r=-1), dict(t=float("inf")),
                dict(anchor=40), dict(anchor=-33), dict(B=2**12, F=2**11)):
        kw = dict(B=2, F=32, H=16, W=16, C=64, dtype=torch.bfloat16, r=1, t=0.7, anchor="auto")
        kw.update(bad)
        with pytest.raises(ttf.TTFError) as e:
            ttf.ttf_workspace_size(**kw)
        assert e.value.status == 1, bad
    # token counts are bounded with every frame rounded up to whole 64-token keep words: below 2^25
    kw = dict(B=2**8, F=2**8, H=1, W=65, C=64, dtype=torch.bfloat16, r=1, t=0.7, anchor="auto")
    assert ttf.ttf_workspace_size(**kw) > 0                      # 2^16 frames x 128 = 2^23
    kw.update(B=2**10)                                           # 2^18 frames x 65 tokens < 2^25, x 128 = 2^25
    with pytest.raises(ttf.TTFError) as e:
        ttf.ttf_workspace_size(**kw)
    assert e.value.status == 1


def test_search_routes():
    """Host-side route query: which window-search kernels a problem takes.  The GPU parity cases that
    are meant for the matrix-core kernels must really be sent there."""
    import torch
    import paper_2605_07355_amd as ttf
    bf, f32 = torch.bfloat16, torch.float32
    route = ttf.ttf_search_route
    assert route(16, 32, 16, 16, 4096, bf, r=1) == "mfma_bf16"
    assert route(4, 64, 32, 32, 4096, bf, r=2) == "mfma_bf16"
    assert route(2, 6, 16, 16, 4000, bf, r=1) == "mfma_bf16"              # whole K-steps, ragged passes
    assert route(2, 6, 14, 14, 128, bf, r=1) == "mfma_bf16_padded"
    assert route(1, 9, 3, 200, 32, bf, r=1) == "mfma_bf16_padded"
    assert route(4, 33, 64, 16, 72, bf, r=2) == "general"                 # C % 32 != 0
    assert route(1, 3, 32, 16, 128, bf, r=3) == "general"                 # radius beyond 5x5
    assert route(16, 32, 16, 16, 4096, f32, r=1) == "mfma_f32"
    assert route(1, 4, 8, 8, 256, f32, r=1) == "general"                  # a handful of workgroups only
    assert route(4, 33, 64, 16, 40, f32, r=1) == "general"
    from test_gpu_parity import F32_MFMA_SHAPES, GRAPH_CASES
    from test_gpu_nonfinite import PATHS
    assert len(F32_MFMA_SHAPES) >= 15
    for B, F, H, W, C, dtype, r in F32_MFMA_SHAPES:
        assert route(B, F, H, W, C, f32, r=r) == "mfma_f32", (B, F, H, W, C, r)
    for name, B, F, H, W, C, dtype, r, spec in list(GRAPH_CASES) + list(PATHS):
        if "fp32" in name and "general" not in name:
            assert route(B, F, H, W, C, f32, r=r) == "mfma_f32", name
        if name.startswith("general"):
            assert route(B, F, H, W, C, f32 if dtype == "f32" else bf, r=r) == "general", name
    # the padded bf16 kernels index a clip's anchor fragments with 32-bit offsets: a grid whose padded
    # frame holds 2^31 elements or more must not reach them
    assert route(1, 2, 1000, 1001, 2048, bf, r=1) == "mfma_bf16_padded"    # 1000 x 1008 x 2048 < 2^31
    assert route(1, 2, 1000, 1001, 4096, bf, r=1) == "general"             # 1000 x 1008 x 4096 >= 2^31
    assert route(1, 2, 1000, 1001, 4096, f32, r=1) == "mfma_f32"           # 64-bit offsets there
    with pytest.raises(ttf.TTFError):
        route(0, 4, 8, 8, 64, bf)


def test_compress_rejects_null_pointers_without_a_gpu():
    """Validation happens before any HIP call, so these return an error code on any machine."""
    import paper_2605_07355_amd as ttf
    from paper_2605_07355_amd import binding
    lib = ttf.load_library()
    p = binding._Params(1, 4, 8, 8, 256, binding.TTF_F32, 1, 0.7, 0, 0)
    o = binding._Outputs()
    assert lib.ttf_compress(None, None, None, 0, None, None) == 1
    assert lib.ttf_compress(ctypes.byref(p), None, None, 0, ctypes.byref(o), None) == 1
    assert lib.ttf_compress(ctypes.byref(p), 4096, 4096, 1 << 30, ctypes.byref(o), None) == 1   # NULL outputs
    p.dtype = 7
    assert lib.ttf_compress(ctypes.byref(p), 4096, 4096, 1 << 30, ctypes.byref(o), None) == 2
    buf = (ctypes.c_float * 6)()
    assert lib.ttf_profile_read(0, buf, 6) == 1         # profiling is off


def test_generator_is_deterministic():
    import numpy as np
    from workloads import CONFIGS, make_clip_batch
    cfg = CONFIGS["qwen3vl_2b"].scaled(B=2, F=4, H=4, W=4, C=32)
    a, b = make_clip_batch(cfg, seed=5), make_clip_batch(cfg, seed=5)
    np.testing.assert_array_equal(a.x, b.x)
    c = make_clip_batch(cfg.scaled(B=1), seed=5)
    np.testing.assert_array_equal(a.x[0], c.x[0])          # clip b depends on (seed, b) only
    assert not np.array_equal(a.x, make_clip_batch(cfg, seed=6).x)


def test_header_is_plain_c(tmp_path):
    """include/ttf.h must be usable from C: compile a translation unit that only includes it."""
    import subprocess
    src = tmp_path / "use_ttf.c"
    src.write_text('#include "ttf.h"\n'
                   'int probe(void) { ttf_params p; ttf_outputs o; (void)p; (void)o;\n'
                   '  return (int)sizeof(ttf_params) + (int)sizeof(ttf_outputs) + TTF_NUM_STAGES; }\n')
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-c", str(src),
                    "-I", os.path.join(ROOT, "include"), "-o", str(tmp_path / "use_ttf.o")], check=True)


def test_struct_layout_matches_binding():
    """The ctypes mirrors must have the sizes the C compiler gives the header's structs."""
    import subprocess, tempfile
    from paper_2605_07355_amd import binding
    with tempfile.TemporaryDirectory() as d:
        src = os.path.join(d, "sz.c")
        with open(src, "w") as fh:
            fh.write('#include <stdio.h>\n#include <stddef.h>\n#include "ttf.h"\n'
                     'int main(void) { printf("%zu %zu %zu %zu\\n", sizeof(ttf_params), sizeof(ttf_outputs),\n'
                     '  offsetof(ttf_params, t), offsetof(ttf_outputs, host_counts)); return 0; }\n')
        exe = os.path.join(d, "sz")
        subprocess.run(["gcc", "-std=c99", src, "-I", os.path.join(ROOT, "include"), "-o", exe], check=True)
        out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout.split()
    assert int(out[0]) == ctypes.sizeof(binding._Params)
    assert int(out[1]) == ctypes.sizeof(binding._Outputs)
    assert int(out[2]) == binding._Params.t.offset
    assert int(out[3]) == binding._Outputs.host_counts.offset
