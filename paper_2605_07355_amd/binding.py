"""ctypes binding of ``include/ttf.h``: same names, argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Union

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG_DIR, "libttf.so")

TTF_OK, TTF_ERR_INVALID_ARG, TTF_ERR_UNSUPPORTED, TTF_ERR_WORKSPACE_TOO_SMALL, TTF_ERR_HIP = range(5)
TTF_BF16, TTF_F32 = 0, 1
TTF_ANCHOR_AUTO, TTF_ANCHOR_FIXED = 0, 1
TTF_NUM_STAGES = 7


class TTFError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"ttf status {status}: {message}")
        self.status = status


class _Params(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("F", ctypes.c_int32), ("H", ctypes.c_int32), ("W", ctypes.c_int32),
                ("C", ctypes.c_int32), ("dtype", ctypes.c_int32), ("r", ctypes.c_int32), ("t", ctypes.c_float),
                ("anchor_mode", ctypes.c_int32), ("anchor_index", ctypes.c_int32)]


class _Outputs(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("tokens_out", "pos_ids", "src_index", "row_offsets", "kept_count", "anchor_index",
                 "fuse_map", "best_sim", "best_idx", "host_counts")]


class _TiedOutputs(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("tokens_out", "pos_ids", "src_index", "kept_count", "anchor_index", "fuse_map",
                 "best_sim", "best_idx", "mean_sim", "host_counts")]


_lib: Optional[ctypes.CDLL] = None


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load ``libttf.so`` from the package directory.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} not found: build it with `python -m paper_2605_07355_amd.build` "
                "(there is no fallback implementation)")
        lib = ctypes.CDLL(_LIB_PATH)
        lib.ttf_workspace_size.restype = ctypes.c_int
        lib.ttf_workspace_size.argtypes = [ctypes.POINTER(_Params), ctypes.POINTER(ctypes.c_size_t)]
        lib.ttf_compress.restype = ctypes.c_int
        lib.ttf_compress.argtypes = [ctypes.POINTER(_Params), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                     ctypes.POINTER(_Outputs), ctypes.c_void_p]
        vp, i64 = ctypes.c_void_p, ctypes.c_int64
        lib.ttf_compress_static.restype = ctypes.c_int
        lib.ttf_compress_static.argtypes = [ctypes.POINTER(_Params), vp, ctypes.POINTER(_Outputs), vp]
        lib.ttf_compress_segment.restype = ctypes.c_int
        lib.ttf_compress_segment.argtypes = [ctypes.POINTER(_Params), vp, vp, ctypes.c_int32, vp, ctypes.c_size_t,
                                             ctypes.POINTER(_Outputs), vp]
        lib.ttf_tied_workspace_size.restype = ctypes.c_int
        lib.ttf_tied_workspace_size.argtypes = [ctypes.POINTER(_Params), ctypes.POINTER(ctypes.c_size_t)]
        lib.ttf_compress_tied.restype = ctypes.c_int
        lib.ttf_compress_tied.argtypes = [ctypes.POINTER(_Params), vp, vp, ctypes.c_size_t,
                                          ctypes.POINTER(_TiedOutputs), vp]
        lib.ttf_restore_map.restype = ctypes.c_int
        lib.ttf_restore_map.argtypes = [ctypes.POINTER(_Params), vp, vp, vp, vp, vp]
        lib.ttf_restore.restype = ctypes.c_int
        lib.ttf_restore.argtypes = [ctypes.POINTER(_Params), vp, i64, vp, vp, vp]
        lib.ttf_decode_alignment.restype = ctypes.c_int
        lib.ttf_decode_alignment.argtypes = [i64, i64, i64] + [ctypes.POINTER(i64)] * 3
        lib.ttf_select_threshold.restype = ctypes.c_int
        lib.ttf_select_threshold.argtypes = [ctypes.POINTER(_Params), vp, vp, ctypes.c_float, vp, vp]
        lib.ttf_regate.restype = ctypes.c_int
        lib.ttf_regate.argtypes = [ctypes.POINTER(_Params), vp, vp, vp, ctypes.c_size_t,
                                   ctypes.POINTER(_Outputs), vp]
        lib.ttf_search_route.restype = ctypes.c_int
        lib.ttf_search_route.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_int)]
        lib.ttf_set_speculation.restype = ctypes.c_int
        lib.ttf_set_speculation.argtypes = [ctypes.c_int]
        lib.ttf_status_string.restype = ctypes.c_char_p
        lib.ttf_status_string.argtypes = [ctypes.c_int]
        lib.ttf_last_hip_error.restype = ctypes.c_int
        lib.ttf_profile_enable.restype = ctypes.c_int
        lib.ttf_profile_enable.argtypes = [ctypes.c_int]
        lib.ttf_profile_read.restype = ctypes.c_int
        lib.ttf_profile_read.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_float), ctypes.c_int]
        lib.ttf_stage_name.restype = ctypes.c_char_p
        lib.ttf_stage_name.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def ttf_status_string(status: int) -> str:
    return load_library().ttf_status_string(int(status)).decode()


def ttf_last_hip_error() -> int:
    return int(load_library().ttf_last_hip_error())


def _check(status: int) -> None:
    if status != TTF_OK:
        raise TTFError(status, ttf_status_string(status))


def _stage_names():
    try:
        lib = load_library()
    except (FileNotFoundError, OSError, AttributeError):   # not built yet, or an older build
        return tuple(f"stage{i}" for i in range(TTF_NUM_STAGES))
    return tuple(lib.ttf_stage_name(i).decode() for i in range(TTF_NUM_STAGES))


STAGE_NAMES = _stage_names()


def _dtype_code(dt: torch.dtype) -> int:
    if dt == torch.bfloat16:
        return TTF_BF16
    if dt == torch.float32:
        return TTF_F32
    raise TypeError(f"features must be bfloat16 or float32, got {dt}")


def _make_params(B, F, H, W, C, dtype_code, r, t, anchor) -> _Params:
    if isinstance(anchor, str):
        if anchor != "auto":
            raise ValueError("anchor must be 'auto' or a frame index")
        mode, idx = TTF_ANCHOR_AUTO, 0
    else:
        mode, idx = TTF_ANCHOR_FIXED, int(anchor)
    return _Params(int(B), int(F), int(H), int(W), int(C), int(dtype_code), int(r), float(t), mode, idx)


def ttf_workspace_size(B: int, F: int, H: int, W: int, C: int, dtype: torch.dtype = torch.bfloat16,
                       r: int = 1, t: float = 0.7, anchor: Union[str, int] = "auto") -> int:
    p = _make_params(B, F, H, W, C, _dtype_code(dtype), r, t, anchor)
    n = ctypes.c_size_t(0)
    _check(load_library().ttf_workspace_size(ctypes.byref(p), ctypes.byref(n)))
    return int(n.value)


@dataclass
class TTFBuffers:
    """Caller-owned device buffers of one problem size, reusable across calls."""
    tokens_out: torch.Tensor     # [cap, C]
    pos_ids: torch.Tensor        # [3, cap] int32
    src_index: torch.Tensor      # [cap] int32
    row_offsets: torch.Tensor    # [B+1] int32
    kept_count: torch.Tensor     # [B] int32
    anchor_index: torch.Tensor   # [B] int32
    fuse_map: torch.Tensor       # [B,F,N] int32
    best_sim: Optional[torch.Tensor]   # [B,F,N] float32
    best_idx: Optional[torch.Tensor]   # [B,F,N] int32
    workspace: torch.Tensor      # uint8
    host_counts: Optional[torch.Tensor] = None   # pinned int32 [2B+1]

    @staticmethod
    def allocate(B, F, H, W, C, dtype, device, want_sim=True, want_host_counts=False) -> "TTFBuffers":
        N, cap = H * W, B * F * H * W
        i32 = dict(dtype=torch.int32, device=device)
        ws = ttf_workspace_size(B, F, H, W, C, dtype)
        return TTFBuffers(
            tokens_out=torch.empty((cap, C), dtype=dtype, device=device),
            pos_ids=torch.empty((3, cap), **i32), src_index=torch.empty((cap,), **i32),
            row_offsets=torch.empty((B + 1,), **i32), kept_count=torch.empty((B,), **i32),
            anchor_index=torch.empty((B,), **i32), fuse_map=torch.empty((B, F, N), **i32),
            best_sim=torch.empty((B, F, N), dtype=torch.float32, device=device) if want_sim else None,
            best_idx=torch.empty((B, F, N), **i32) if want_sim else None,
            workspace=torch.empty((ws + 256,), dtype=torch.uint8, device=device),
            host_counts=torch.empty((2 * B + 1,), dtype=torch.int32, pin_memory=True) if want_host_counts else None)


@dataclass
class TTFOutput:
    buffers: TTFBuffers
    B: int
    F: int
    H: int
    W: int
    C: int

    # views; reading them synchronises as any torch op on the stream does
    @property
    def total_rows(self) -> int:
        return int(self.buffers.row_offsets[-1].item())

    def clip_tokens(self, b: int) -> torch.Tensor:
        ro = self.buffers.row_offsets
        return self.buffers.tokens_out[int(ro[b]):int(ro[b + 1])]

    def clip_pos_ids(self, b: int) -> torch.Tensor:
        ro = self.buffers.row_offsets
        return self.buffers.pos_ids[:, int(ro[b]):int(ro[b + 1])]


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _aligned_workspace(ws: torch.Tensor):
    base = ws.data_ptr()
    off = (-base) % 256
    return base + off, ws.numel() - off


def ttf_compress(features: torch.Tensor, r: int = 1, t: float = 0.70, anchor: Union[str, int] = "auto",
                 buffers: Optional[TTFBuffers] = None, want_sim: bool = True,
                 stream: Optional[torch.cuda.Stream] = None) -> TTFOutput:
    """Run the TTF pass on ``features`` [B,F,H,W,C] (CUDA/HIP tensor, bf16 or fp32, contiguous).

    Enqueues on ``stream`` (default: the current stream) and returns without synchronising.
    ``buffers`` may be passed to reuse allocations; otherwise they are allocated with torch.
    """
    if features.dim() != 5:
        raise ValueError("features must be [B,F,H,W,C]")
    if not features.is_cuda:
        raise ValueError("features must live on the GPU (the library has no CPU path)")
    if not features.is_contiguous():
        raise ValueError("features must be contiguous")
    B, F, H, W, C = (int(v) for v in features.shape)
    p = _make_params(B, F, H, W, C, _dtype_code(features.dtype), r, t, anchor)
    if buffers is None:
        buffers = TTFBuffers.allocate(B, F, H, W, C, features.dtype, features.device, want_sim=want_sim)
    ws_ptr, ws_bytes = _aligned_workspace(buffers.workspace)
    o = _Outputs(_ptr(buffers.tokens_out), _ptr(buffers.pos_ids), _ptr(buffers.src_index),
                 _ptr(buffers.row_offsets), _ptr(buffers.kept_count), _ptr(buffers.anchor_index),
                 _ptr(buffers.fuse_map), _ptr(buffers.best_sim), _ptr(buffers.best_idx),
                 _ptr(buffers.host_counts))
    s = stream if stream is not None else torch.cuda.current_stream(features.device)
    with torch.cuda.device(features.device):
        _check(load_library().ttf_compress(ctypes.byref(p), features.data_ptr(), ws_ptr, ws_bytes,
                                           ctypes.byref(o), ctypes.c_void_p(s.cuda_stream)))
    return TTFOutput(buffers, B, F, H, W, C)


TTF_STATIC_WORKSPACE_BYTES = 16 << 20


def ttf_compress_static(features: torch.Tensor, buffers: TTFBuffers, r: int = 1, t: float = 0.70,
                        anchor: Union[str, int] = "auto",
                        stream: Optional[torch.cuda.Stream] = None) -> TTFOutput:
    """``ttf_compress`` on the library's built-in workspace: nothing is allocated by the call, so
    ``buffers`` (outputs; its ``workspace`` field is not used) must be given.  Problems that need more
    than ``TTF_STATIC_WORKSPACE_BYTES`` of workspace raise ``TTFError`` (status 3)."""
    if features.dim() != 5 or not features.is_cuda or not features.is_contiguous():
        raise ValueError("features must be a contiguous [B,F,H,W,C] GPU tensor")
    B, F, H, W, C = (int(v) for v in features.shape)
    p = _make_params(B, F, H, W, C, _dtype_code(features.dtype), r, t, anchor)
    o = _outputs_of(buffers)
    with torch.cuda.device(features.device):
        _check(load_library().ttf_compress_static(ctypes.byref(p), features.data_ptr(), ctypes.byref(o),
                                                  _stream_ptr(stream, features.device)))
    return TTFOutput(buffers, B, F, H, W, C)


def _stream_ptr(stream, device):
    s = stream if stream is not None else torch.cuda.current_stream(device)
    return ctypes.c_void_p(s.cuda_stream)


def _outputs_of(buffers: TTFBuffers) -> _Outputs:
    return _Outputs(_ptr(buffers.tokens_out), _ptr(buffers.pos_ids), _ptr(buffers.src_index),
                    _ptr(buffers.row_offsets), _ptr(buffers.kept_count), _ptr(buffers.anchor_index),
                    _ptr(buffers.fuse_map), _ptr(buffers.best_sim), _ptr(buffers.best_idx),
                    _ptr(buffers.host_counts))


def ttf_compress_segment(features: torch.Tensor, anchor_frame: torch.Tensor, frame_offset: int = 0,
                         r: int = 1, t: float = 0.70, buffers: Optional[TTFBuffers] = None,
                         want_sim: bool = True, stream: Optional[torch.cuda.Stream] = None) -> TTFOutput:
    """One stream segment ``features`` [B,F,H,W,C] against the rolling ``anchor_frame`` [B,H,W,C]:
    only preserved source rows are emitted; temporal ids start at ``frame_offset``."""
    if features.dim() != 5 or not features.is_cuda or not features.is_contiguous():
        raise ValueError("features must be a contiguous [B,F,H,W,C] GPU tensor")
    B, F, H, W, C = (int(v) for v in features.shape)
    if (tuple(anchor_frame.shape) != (B, H, W, C) or anchor_frame.dtype != features.dtype
            or anchor_frame.device != features.device or not anchor_frame.is_contiguous()):
        raise ValueError("anchor_frame must be a contiguous [B,H,W,C] tensor like one frame of features")
    p = _make_params(B, F, H, W, C, _dtype_code(features.dtype), r, t, "auto")
    if buffers is None:
        buffers = TTFBuffers.allocate(B, F, H, W, C, features.dtype, features.device, want_sim=want_sim)
    ws_ptr, ws_bytes = _aligned_workspace(buffers.workspace)
    o = _outputs_of(buffers)
    with torch.cuda.device(features.device):
        _check(load_library().ttf_compress_segment(ctypes.byref(p), features.data_ptr(), anchor_frame.data_ptr(),
                                                   int(frame_offset), ws_ptr, ws_bytes, ctypes.byref(o),
                                                   _stream_ptr(stream, features.device)))
    return TTFOutput(buffers, B, F, H, W, C)


@dataclass
class TTFTiedBuffers:
    """Caller-owned device buffers of the tied-batch mode."""
    tokens_out: torch.Tensor     # [B, F*N, C]
    pos_ids: torch.Tensor        # [3, F*N] int32
    src_index: torch.Tensor      # [F*N] int32
    kept_count: torch.Tensor     # [1] int32
    anchor_index: torch.Tensor   # [B] int32
    fuse_map: torch.Tensor       # [F,N] int32
    best_sim: Optional[torch.Tensor]   # [B,F,N] float32
    best_idx: Optional[torch.Tensor]   # [F,N] int32
    mean_sim: Optional[torch.Tensor]   # [F,N] float32
    workspace: torch.Tensor

    @staticmethod
    def allocate(B, F, H, W, C, dtype, device, r=1, want_sim=True) -> "TTFTiedBuffers":
        N = H * W
        i32 = dict(dtype=torch.int32, device=device)
        f32 = dict(dtype=torch.float32, device=device)
        return TTFTiedBuffers(
            tokens_out=torch.empty((B, F * N, C), dtype=dtype, device=device),
            pos_ids=torch.empty((3, F * N), **i32), src_index=torch.empty((F * N,), **i32),
            kept_count=torch.empty((1,), **i32), anchor_index=torch.empty((B,), **i32),
            fuse_map=torch.empty((F, N), **i32),
            best_sim=torch.empty((B, F, N), **f32) if want_sim else None,
            best_idx=torch.empty((F, N), **i32) if want_sim else None,
            mean_sim=torch.empty((F, N), **f32) if want_sim else None,
            workspace=torch.empty((ttf_tied_workspace_size(B, F, H, W, C, dtype, r) + 256,),
                                  dtype=torch.uint8, device=device))


def ttf_tied_workspace_size(B: int, F: int, H: int, W: int, C: int, dtype: torch.dtype = torch.bfloat16,
                            r: int = 1) -> int:
    p = _make_params(B, F, H, W, C, _dtype_code(dtype), r, 0.7, "auto")
    n = ctypes.c_size_t(0)
    _check(load_library().ttf_tied_workspace_size(ctypes.byref(p), ctypes.byref(n)))
    return int(n.value)


def ttf_compress_tied(features: torch.Tensor, r: int = 1, t: float = 0.70, anchor: Union[str, int] = "auto",
                      buffers: Optional[TTFTiedBuffers] = None, want_sim: bool = True,
                      stream: Optional[torch.cuda.Stream] = None) -> TTFTiedBuffers:
    """Tied-batch pass on ``features`` [B,F,H,W,C]: one shared offset and one shared keep mask for
    all B elements; rectangular output (see ``TTFTiedBuffers``)."""
    if features.dim() != 5 or not features.is_cuda or not features.is_contiguous():
        raise ValueError("features must be a contiguous [B,F,H,W,C] GPU tensor")
    B, F, H, W, C = (int(v) for v in features.shape)
    p = _make_params(B, F, H, W, C, _dtype_code(features.dtype), r, t, anchor)
    if buffers is None:
        buffers = TTFTiedBuffers.allocate(B, F, H, W, C, features.dtype, features.device, r=r, want_sim=want_sim)
    ws_ptr, ws_bytes = _aligned_workspace(buffers.workspace)
    o = _TiedOutputs(_ptr(buffers.tokens_out), _ptr(buffers.pos_ids), _ptr(buffers.src_index),
                     _ptr(buffers.kept_count), _ptr(buffers.anchor_index), _ptr(buffers.fuse_map),
                     _ptr(buffers.best_sim), _ptr(buffers.best_idx), _ptr(buffers.mean_sim), None)
    with torch.cuda.device(features.device):
        _check(load_library().ttf_compress_tied(ctypes.byref(p), features.data_ptr(), ws_ptr, ws_bytes,
                                                ctypes.byref(o), _stream_ptr(stream, features.device)))
    return buffers


def ttf_restore_map(out: TTFOutput, restore_map: Optional[torch.Tensor] = None,
                    stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """int32 [B,F,N]: the compressed row that stands for every original token."""
    b = out.buffers
    dev = b.fuse_map.device
    if restore_map is None:
        restore_map = torch.empty((out.B, out.F, out.H * out.W), dtype=torch.int32, device=dev)
    p = _make_params(out.B, out.F, out.H, out.W, out.C, _dtype_code(b.tokens_out.dtype), 0, 0.0, "auto")
    with torch.cuda.device(dev):
        _check(load_library().ttf_restore_map(ctypes.byref(p), b.fuse_map.data_ptr(), b.row_offsets.data_ptr(),
                                              b.src_index.data_ptr(), restore_map.data_ptr(),
                                              _stream_ptr(stream, dev)))
    return restore_map


def ttf_restore(tokens: torch.Tensor, rows: int, restore_map: torch.Tensor, H: int, W: int,
                restored: Optional[torch.Tensor] = None,
                stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """[B,F,H,W,C]: ``tokens[restore_map]`` -- the full layout rebuilt from compressed rows."""
    B, F, N = (int(v) for v in restore_map.shape)
    C = int(tokens.shape[-1])
    if N != H * W:
        raise ValueError("restore_map does not match the grid")
    if not tokens.is_contiguous() or not restore_map.is_contiguous() or restore_map.dtype != torch.int32:
        raise ValueError("tokens and restore_map must be contiguous, restore_map int32")
    if rows > tokens.shape[0]:
        raise ValueError("rows exceeds the token buffer")
    if restored is None:
        restored = torch.empty((B, F, H, W, C), dtype=tokens.dtype, device=tokens.device)
    p = _make_params(B, F, H, W, C, _dtype_code(tokens.dtype), 0, 0.0, "auto")
    with torch.cuda.device(tokens.device):
        _check(load_library().ttf_restore(ctypes.byref(p), tokens.data_ptr(), int(rows), restore_map.data_ptr(),
                                          restored.data_ptr(), _stream_ptr(stream, tokens.device)))
    return restored


def ttf_decode_alignment(l_prime: int, text_tokens: int, step: int):
    """(L_pre, position of decode step ``step``, attention-mask length at that step)."""
    v = [ctypes.c_int64(0) for _ in range(3)]
    _check(load_library().ttf_decode_alignment(int(l_prime), int(text_tokens), int(step),
                                               *(ctypes.byref(x) for x in v)))
    return tuple(int(x.value) for x in v)


def ttf_select_threshold(out: TTFOutput, fused_fraction: float, thresholds: Optional[torch.Tensor] = None,
                         stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """float32 [B]: per-clip threshold that fuses at most ``fused_fraction`` of the source tokens."""
    b = out.buffers
    if b.best_sim is None:
        raise ValueError("threshold selection needs best_sim (want_sim=True)")
    dev = b.best_sim.device
    if thresholds is None:
        thresholds = torch.empty((out.B,), dtype=torch.float32, device=dev)
    p = _make_params(out.B, out.F, out.H, out.W, out.C, _dtype_code(b.tokens_out.dtype), 0, 0.0, "auto")
    with torch.cuda.device(dev):
        _check(load_library().ttf_select_threshold(ctypes.byref(p), b.best_sim.data_ptr(),
                                                   b.anchor_index.data_ptr(), float(fused_fraction),
                                                   thresholds.data_ptr(), _stream_ptr(stream, dev)))
    return thresholds


def ttf_regate(features: torch.Tensor, out: TTFOutput, thresholds: Optional[torch.Tensor] = None,
               t: float = 0.70, stream: Optional[torch.cuda.Stream] = None) -> TTFOutput:
    """Redo gate, offsets and rows of ``out`` (in place) from its stored matches, at per-clip
    ``thresholds`` (float32 [B] on the GPU) or at ``t`` for every clip."""
    b = out.buffers
    if b.best_sim is None or b.best_idx is None:
        raise ValueError("regating needs best_sim and best_idx (want_sim=True)")
    if tuple(features.shape) != (out.B, out.F, out.H, out.W, out.C) or not features.is_contiguous():
        raise ValueError("features must be the contiguous tensor the matches were computed from")
    if thresholds is not None and (thresholds.dtype != torch.float32 or thresholds.numel() != out.B
                                   or not thresholds.is_cuda):
        raise ValueError("thresholds must be float32 [B] on the GPU")
    p = _make_params(out.B, out.F, out.H, out.W, out.C, _dtype_code(features.dtype), 0, t, "auto")
    ws_ptr, ws_bytes = _aligned_workspace(b.workspace)
    o = _outputs_of(b)
    with torch.cuda.device(features.device):
        _check(load_library().ttf_regate(ctypes.byref(p), features.data_ptr(), _ptr(thresholds), ws_ptr, ws_bytes,
                                         ctypes.byref(o), _stream_ptr(stream, features.device)))
    return out


ROUTE_NAMES = {0: "general", 1: "mfma_bf16", 2: "mfma_bf16_padded", 3: "mfma_f32"}


def ttf_search_route(B: int, F: int, H: int, W: int, C: int, dtype: torch.dtype = torch.bfloat16,
                     r: int = 1, t: float = 0.7, anchor: Union[str, int] = "auto") -> str:
    """Name of the window-search kernels this problem takes (see ROUTE_NAMES); host-side query."""
    p = _make_params(B, F, H, W, C, _dtype_code(dtype), r, t, anchor)
    route = ctypes.c_int(-1)
    _check(load_library().ttf_search_route(ctypes.byref(p), ctypes.byref(route)))
    return ROUTE_NAMES[int(route.value)]


def ttf_set_speculation(mode: int) -> None:
    """How the automatic anchor rule is evaluated: 0 speculative single pass for large inputs where
    available (default), 1 wherever available, -1 always the two-pass route.  Outputs never differ."""
    _check(load_library().ttf_set_speculation(int(mode)))


def ttf_profile_enable(slots: int) -> None:
    """Record per-stage HIP events for the following calls (``slots`` event sets, 0 = off)."""
    _check(load_library().ttf_profile_enable(int(slots)))


def ttf_profile_read(call: int = 0):
    """Stage durations (ms) of profiled call number ``call`` on this thread, keyed by stage name."""
    buf = (ctypes.c_float * TTF_NUM_STAGES)()
    _check(load_library().ttf_profile_read(int(call), buf, TTF_NUM_STAGES))
    return {STAGE_NAMES[i]: float(buf[i]) for i in range(TTF_NUM_STAGES)}
