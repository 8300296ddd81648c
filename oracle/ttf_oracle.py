"""ctypes front-end of the CPU oracle (``ttf_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may import this
module.  It shares nothing with the GPU library.  ``build()`` compiles the C file with gcc
into ``libttf_oracle.so`` next to it; loading builds on demand when the library is absent.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ttf_oracle.c")
_LIB = os.path.join(_HERE, "libttf_oracle.so")

BF16, F32 = 0, 1
ANCHOR_AUTO, ANCHOR_FIXED = 0, 1

_lib: Optional[ctypes.CDLL] = None

# code-generation flags of the oracle library (reported next to its timing)
BUILD_FLAGS = ("-O2", "-std=c11", "-fopenmp", "-ffp-contract=off")


def build(force: bool = True) -> str:
    """Compile the oracle.  Portable flags on purpose: the library is built on one machine
    and may run on another; no fast-math and no contraction, so every operation is the
    plain IEEE double one the source spells out."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", *BUILD_FLAGS, "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        vp, ip, dp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_double)
        ci = ctypes.c_int
        lib.ttf_oracle_threads.restype = ci
        lib.ttf_oracle_compress.restype = ci
        lib.ttf_oracle_compress.argtypes = [vp, ci, ci, ci, ci, ci, ci, ci, ctypes.c_float, ci, ci,
                                            ip, dp, dp, dp, ip, ip, ip, ip, ip, ip, ip, vp]
        lib.ttf_oracle_compress_tied.restype = ci
        lib.ttf_oracle_compress_tied.argtypes = [vp, ci, ci, ci, ci, ci, ci, ci, ctypes.c_float, ci, ci,
                                                 ip, dp, dp, dp, dp, ip, ip, ip, ip, ip, vp]
        lib.ttf_oracle_match_tokens.restype = ci
        lib.ttf_oracle_match_tokens.argtypes = [vp, ci, ci, ci, ci, ci, ci, ci, ip, ip, ci, dp, dp, ip]
        _lib = lib
    return _lib


def threads() -> int:
    return int(_load().ttf_oracle_threads())


def _dtype_code(x: np.ndarray) -> int:
    if x.dtype == np.float32:
        return F32
    if x.dtype == np.uint16:
        return BF16
    raise TypeError("oracle input must be float32 or uint16 (bf16 bit patterns)")


def _ip(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _dp(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


@dataclass
class OracleResult:
    anchor_index: np.ndarray   # [B]       int32
    anchor_score: np.ndarray   # [B,F]     float64
    best_sim: np.ndarray       # [B,F,N]   float64
    second_sim: np.ndarray     # [B,F,N]   float64
    best_idx: np.ndarray       # [B,F,N]   int32
    cand_count: np.ndarray     # [B,F,N]   int32
    fuse_map: np.ndarray       # [B,F,N]   int32
    kept_count: np.ndarray     # [B]       int32
    row_offsets: np.ndarray    # [B+1]     int32
    src_index: np.ndarray      # [cap]     int32 (valid up to row_offsets[B])
    pos_ids: np.ndarray        # [3,cap]   int32
    tokens_out: Optional[np.ndarray]  # [cap,C] input dtype, or None

    @property
    def total_rows(self) -> int:
        return int(self.row_offsets[-1])

    def fused_fraction(self) -> float:
        B, F, N = self.fuse_map.shape
        return float((self.fuse_map >= 0).sum()) / float(max(1, B * (F - 1) * N))

    def reduction_ratio(self) -> np.ndarray:
        """rho = 1 - (N+P)/(F N) per clip (Section 3, after the stacked X')."""
        B, F, N = self.fuse_map.shape
        return 1.0 - self.kept_count.astype(np.float64) / float(F * N)


def compress(x: np.ndarray, r: int, t: float, anchor_mode: int = ANCHOR_AUTO,
             anchor_index: int = 0, want_tokens: bool = True) -> OracleResult:
    """Run the whole pass on ``x`` [B,F,H,W,C] (float32, or uint16 bf16 bits)."""
    if x.ndim != 5:
        raise ValueError("x must be [B,F,H,W,C]")
    x = np.ascontiguousarray(x)
    B, F, H, W, C = (int(v) for v in x.shape)
    N, cap = H * W, B * F * H * W
    res = OracleResult(
        anchor_index=np.zeros(B, np.int32), anchor_score=np.zeros((B, F), np.float64),
        best_sim=np.zeros((B, F, N), np.float64), second_sim=np.zeros((B, F, N), np.float64),
        best_idx=np.zeros((B, F, N), np.int32), cand_count=np.zeros((B, F, N), np.int32),
        fuse_map=np.zeros((B, F, N), np.int32), kept_count=np.zeros(B, np.int32),
        row_offsets=np.zeros(B + 1, np.int32), src_index=np.full(cap, -1, np.int32),
        pos_ids=np.full((3, cap), -1, np.int32),
        tokens_out=np.zeros((cap, C), x.dtype) if want_tokens else None)
    rc = _load().ttf_oracle_compress(
        x.ctypes.data, _dtype_code(x), B, F, H, W, C, int(r), float(np.float32(t)),
        int(anchor_mode), int(anchor_index),
        _ip(res.anchor_index), _dp(res.anchor_score), _dp(res.best_sim), _dp(res.second_sim),
        _ip(res.best_idx), _ip(res.cand_count), _ip(res.fuse_map), _ip(res.kept_count),
        _ip(res.row_offsets), _ip(res.src_index), _ip(res.pos_ids),
        res.tokens_out.ctypes.data if want_tokens else None)
    if rc != 0:
        raise ValueError("ttf_oracle_compress rejected its arguments")
    return res


def match_tokens(x: np.ndarray, r: int, anchor_index: Sequence[int], tokens: np.ndarray):
    """Window search for selected tokens.  ``tokens`` is [n,3] of (b,k,i).  Returns
    (best_sim f64 [n], second_sim f64 [n], best_idx i32 [n])."""
    x = np.ascontiguousarray(x)
    B, F, H, W, C = (int(v) for v in x.shape)
    tok = np.ascontiguousarray(tokens, dtype=np.int32).reshape(-1, 3)
    anc = np.ascontiguousarray(anchor_index, dtype=np.int32)
    n = tok.shape[0]
    best = np.zeros(n, np.float64)
    second = np.zeros(n, np.float64)
    idx = np.zeros(n, np.int32)
    rc = _load().ttf_oracle_match_tokens(x.ctypes.data, _dtype_code(x), B, F, H, W, C, int(r),
                                         _ip(anc), _ip(tok), n, _dp(best), _dp(second), _ip(idx))
    if rc != 0:
        raise ValueError("ttf_oracle_match_tokens rejected its arguments")
    return best, second, idx


@dataclass
class TiedResult:
    anchor_index: int          # shared anchor frame
    anchor_score: np.ndarray   # [F]      batch-mean anchor score
    mean_sim: np.ndarray       # [F,N]    largest batch-mean similarity
    second_mean: np.ndarray    # [F,N]    runner-up batch-mean similarity
    best_sim: np.ndarray       # [B,F,N]  per-element s^ at the shared offset
    best_idx: np.ndarray       # [F,N]    shared dst
    fuse_map: np.ndarray       # [F,N]
    kept_count: int            # L'
    src_index: np.ndarray      # [F*N]
    pos_ids: np.ndarray        # [3,F*N]
    tokens_out: Optional[np.ndarray]   # [B,F*N,C]


def compress_tied(x: np.ndarray, r: int, t: float, anchor_mode: int = ANCHOR_AUTO,
                  anchor_index: int = 0, want_tokens: bool = True) -> TiedResult:
    """The tied-batch pass on ``x`` [B,F,H,W,C]: one offset per position from the batch-mean
    similarity, keep masks united over the batch, rectangular output."""
    x = np.ascontiguousarray(x)
    B, F, H, W, C = (int(v) for v in x.shape)
    N = H * W
    a = np.zeros(1, np.int32)
    kept = np.zeros(1, np.int32)
    res = TiedResult(
        anchor_index=0, anchor_score=np.zeros(F, np.float64), mean_sim=np.zeros((F, N), np.float64),
        second_mean=np.zeros((F, N), np.float64), best_sim=np.zeros((B, F, N), np.float64),
        best_idx=np.zeros((F, N), np.int32), fuse_map=np.zeros((F, N), np.int32), kept_count=0,
        src_index=np.full(F * N, -1, np.int32), pos_ids=np.full((3, F * N), -1, np.int32),
        tokens_out=np.zeros((B, F * N, C), x.dtype) if want_tokens else None)
    rc = _load().ttf_oracle_compress_tied(
        x.ctypes.data, _dtype_code(x), B, F, H, W, C, int(r), float(np.float32(t)),
        int(anchor_mode), int(anchor_index), _ip(a), _dp(res.anchor_score), _dp(res.mean_sim),
        _dp(res.second_mean), _dp(res.best_sim), _ip(res.best_idx), _ip(res.fuse_map), _ip(kept),
        _ip(res.src_index), _ip(res.pos_ids), res.tokens_out.ctypes.data if want_tokens else None)
    if rc != 0:
        raise ValueError("ttf_oracle_compress_tied rejected its arguments")
    res.anchor_index = int(a[0])
    res.kept_count = int(kept[0])
    return res
