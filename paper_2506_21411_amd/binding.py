"""ctypes binding of include/dchag.h.  Argument marshalling only.

Tensors are torch tensors on the current ROCm device (torch is used for device memory and
streams, nothing else); they must be contiguous and of dtype float32 (DCHAG_F32) or
bfloat16 (DCHAG_BF16).  Each function has the name and the meaning of the C entry point.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

DCHAG_F32 = 0
DCHAG_BF16 = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdchag.so")
_lib = None


class DchagError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"dchag status {status}: {message}")
        self.status = status


class _CLevel(ctypes.Structure):
    _fields_ = [("group_size", ctypes.c_int32), ("kind", ctypes.c_int32),
                ("query", ctypes.c_void_p),
                ("Wq", ctypes.c_void_p), ("Wk", ctypes.c_void_p), ("Wv", ctypes.c_void_p), ("Wo", ctypes.c_void_p),
                ("bq", ctypes.c_void_p), ("bk", ctypes.c_void_p), ("bv", ctypes.c_void_p), ("bo", ctypes.c_void_p)]


class _CLevelGrads(ctypes.Structure):
    _fields_ = [("dquery", ctypes.c_void_p),
                ("dWq", ctypes.c_void_p), ("dWk", ctypes.c_void_p), ("dWv", ctypes.c_void_p), ("dWo", ctypes.c_void_p),
                ("dbq", ctypes.c_void_p), ("dbk", ctypes.c_void_p), ("dbv", ctypes.c_void_p), ("dbo", ctypes.c_void_p)]


class _CStageTime(ctypes.Structure):
    _fields_ = [("stage", ctypes.c_int32), ("level", ctypes.c_int32), ("ms", ctypes.c_float)]


STAGE_NAMES = {0: "tokenize", 1: "query", 2: "fold", 3: "scores", 4: "vproj", 5: "softmax_agg", 6: "oproj",
               7: "fused_vagg", 8: "channel_mix", 9: "tokenize_mix", 10: "head_sums", 11: "head_vproj",
               12: "bwd_oproj", 13: "bwd_value", 14: "bwd_softmax", 15: "bwd_tokens", 16: "bwd_key_query",
               17: "bwd_tokenize", 18: "bwd_channel_mix", 19: "fold_value", 20: "tokenize_attend", 21: "key_prep"}

LEVEL_ATTENTION, LEVEL_LINEAR = 0, 1


@dataclass
class LevelWeights:
    """Device tensors of one aggregation level.

    Attention level (kind 0): query [G,D]; Wq..Wo [G,D,D]; biases [G,D] or None.
    Linear level (kind 1, D-CHAG-L): Wv = mixing weights [G,g,D], bv = bias [G,D] or None; the rest None.
    """
    group_size: int
    query: Optional[torch.Tensor]
    Wq: Optional[torch.Tensor]
    Wk: Optional[torch.Tensor]
    Wv: torch.Tensor
    Wo: Optional[torch.Tensor]
    bq: Optional[torch.Tensor] = None
    bk: Optional[torch.Tensor] = None
    bv: Optional[torch.Tensor] = None
    bo: Optional[torch.Tensor] = None
    kind: int = LEVEL_ATTENTION


@dataclass
class LevelGrads:
    """Gradient tensors of one level, shaped like its weights; None = not wanted."""
    dquery: Optional[torch.Tensor] = None
    dWq: Optional[torch.Tensor] = None
    dWk: Optional[torch.Tensor] = None
    dWv: Optional[torch.Tensor] = None
    dWo: Optional[torch.Tensor] = None
    dbq: Optional[torch.Tensor] = None
    dbk: Optional[torch.Tensor] = None
    dbv: Optional[torch.Tensor] = None
    dbo: Optional[torch.Tensor] = None


def library_path() -> str:
    return _LIB_PATH


def use_library(path: str) -> None:
    """Point the binding at another build of the library (the benchmark's timing-probe builds); before the first call."""
    global _LIB_PATH
    if _lib is not None:
        raise RuntimeError("the library is already loaded")
    _LIB_PATH = os.path.abspath(path)


def load_library():
    """Loads libdchag.so (built by `python -m paper_2506_21411_amd.build`); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2506_21411_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(_LIB_PATH)
    i, vp, sz = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
    lib.dchag_tokenize.restype = i
    lib.dchag_tokenize.argtypes = [i] * 7 + [vp] * 6
    lib.dchag_aggregate_level.restype = i
    lib.dchag_aggregate_level.argtypes = [i] * 6 + [ctypes.POINTER(_CLevel), vp, vp, vp, sz, vp]
    lib.dchag_yardstick_mfma.restype = i
    lib.dchag_yardstick_mfma.argtypes = [i, vp, sz, ctypes.POINTER(ctypes.c_double), vp]
    lib.dchag_yardstick_copy.restype = i
    lib.dchag_yardstick_copy.argtypes = [vp, vp, sz, vp]
    lib.dchag_yardstick_read.restype = i
    lib.dchag_yardstick_read.argtypes = [vp, sz, vp, vp]
    lib.dchag_debug_reload.restype = None
    lib.dchag_debug_reload.argtypes = []
    lib.dchag_aggregate_level_static.restype = i
    lib.dchag_aggregate_level_static.argtypes = [i] * 6 + [ctypes.POINTER(_CLevel), vp, vp, vp]
    lib.dchag_forward.restype = i
    lib.dchag_forward.argtypes = [i] * 8 + [vp] * 4 + [i, ctypes.POINTER(_CLevel), vp, vp, sz, vp]
    lib.dchag_forward_pos.restype = i
    lib.dchag_forward_pos.argtypes = [i] * 8 + [vp] * 4 + [i, ctypes.POINTER(_CLevel), vp, vp, vp, sz, vp]
    lib.dchag_forward_folded.restype = i
    lib.dchag_forward_folded.argtypes = lib.dchag_forward.argtypes
    lib.dchag_value_fold_bytes.restype = sz
    lib.dchag_value_fold_bytes.argtypes = [i] * 6 + [ctypes.POINTER(_CLevel)]
    lib.dchag_fold_value.restype = i
    lib.dchag_fold_value.argtypes = [i] * 5 + [vp] * 3 + [i, ctypes.POINTER(_CLevel), vp, sz, vp]
    lib.dchag_forward_prefolded.restype = i
    lib.dchag_forward_prefolded.argtypes = [i] * 8 + [vp] * 4 + [i, ctypes.POINTER(_CLevel), vp, vp, vp, sz, vp]
    lib.dchag_backward.restype = i
    lib.dchag_backward.argtypes = ([i] * 8 + [vp] * 4 + [i, ctypes.POINTER(_CLevel), vp, vp, vp, vp,
                                                        ctypes.POINTER(_CLevelGrads), vp, sz, vp])
    lib.dchag_forward_keep.restype = i
    lib.dchag_forward_keep.argtypes = lib.dchag_forward.argtypes
    lib.dchag_backward_kept.restype = i
    lib.dchag_backward_kept.argtypes = lib.dchag_backward.argtypes
    lib.dchag_workspace_bytes.restype = sz
    lib.dchag_workspace_bytes.argtypes = [i] * 9 + [ctypes.POINTER(ctypes.c_int32), i]
    lib.dchag_strerror.restype = ctypes.c_char_p
    lib.dchag_strerror.argtypes = [i]
    lib.dchag_version.restype = ctypes.c_char_p
    lib.dchag_profile_begin.restype = i
    lib.dchag_profile_end.restype = i
    lib.dchag_profile_end.argtypes = [ctypes.POINTER(_CStageTime), i]
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != 0:
        raise DchagError(status, load_library().dchag_strerror(status).decode())


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return DCHAG_F32
    if t.dtype == torch.bfloat16:
        return DCHAG_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t: Optional[torch.Tensor], like: Optional[torch.Tensor] = None):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous device tensors")
    if like is not None and t.dtype != like.dtype:
        raise TypeError("all tensors of a call must share one dtype")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _clevel(lv: LevelWeights, like: torch.Tensor) -> _CLevel:
    c = _CLevel()
    c.group_size = int(lv.group_size)
    c.kind = int(lv.kind)
    for name in ("query", "Wq", "Wk", "Wv", "Wo", "bq", "bk", "bv", "bo"):
        setattr(c, name, _ptr(getattr(lv, name), like))
    return c


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def dchag_workspace_bytes(dt: int, B: int, C: int, H: int, W: int, p: int, D: int, heads: int,
                          group_sizes: Sequence[int], which: int) -> int:
    arr = (ctypes.c_int32 * len(group_sizes))(*[int(g) for g in group_sizes])
    return int(load_library().dchag_workspace_bytes(dt, B, C, H, W, p, D, heads, len(group_sizes), arr, which))


def dchag_tokenize(x: torch.Tensor, We: torch.Tensor, be: Optional[torch.Tensor], ce: Optional[torch.Tensor],
                   p: int, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """tokens[B,C,N,D] of x[B,C,H,W] with We[C,D,p*p], be/ce [C,D] or None."""
    B, C, H, W = x.shape
    D = We.shape[1]
    if tuple(We.shape) != (C, D, p * p):
        raise ValueError("We must be [C, D, p*p]")
    N = (H // p) * (W // p) if p > 0 else 0
    if out is None:
        out = torch.empty((B, C, N, D), dtype=x.dtype, device=x.device)
    _check(load_library().dchag_tokenize(_dt(x), B, C, H, W, p, D, _ptr(x), _ptr(We, x), _ptr(be, x), _ptr(ce, x),
                                         _ptr(out, x), _stream(stream)))
    return out


def dchag_aggregate_level(tokens_in: torch.Tensor, level: LevelWeights, heads: int,
                          out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                          stream=None) -> torch.Tensor:
    """tokens_out[B,G,N,D] of tokens_in[B,Cin,N,D] for one level."""
    B, Cin, N, D = tokens_in.shape
    g = int(level.group_size)
    G = (Cin + g - 1) // g if g > 0 else 0
    dt = _dt(tokens_in)
    if workspace is None:
        workspace = _workspace(dchag_workspace_bytes(dt, B, Cin, N, 1, 1, D, heads, [g], 0), tokens_in.device)
    if out is None:
        out = torch.empty((B, G, N, D), dtype=tokens_in.dtype, device=tokens_in.device)
    cl = _clevel(level, tokens_in)
    _check(load_library().dchag_aggregate_level(dt, B, Cin, N, D, heads, ctypes.byref(cl), _ptr(tokens_in),
                                                _ptr(out, tokens_in), ctypes.c_void_p(workspace.data_ptr()),
                                                workspace.numel(), _stream(stream)))
    return out


STATIC_SCRATCH_BYTES = 32 << 20


def dchag_aggregate_level_static(tokens_in: torch.Tensor, level: LevelWeights, heads: int, out: torch.Tensor,
                                 stream=None) -> torch.Tensor:
    """dchag_aggregate_level on the library's fixed scratch array: no workspace argument, nothing allocated (the
    caller passes `out`)."""
    B, Cin, N, D = tokens_in.shape
    cl = _clevel(level, tokens_in)
    _check(load_library().dchag_aggregate_level_static(_dt(tokens_in), B, Cin, N, D, heads, ctypes.byref(cl),
                                                       _ptr(tokens_in), _ptr(out, tokens_in), _stream(stream)))
    return out


def dchag_debug_reload() -> None:
    """Re-read the DCHAG_* debugging switches from the environment (the library reads them once, at load)."""
    load_library().dchag_debug_reload()


def dchag_forward(x: torch.Tensor, We: torch.Tensor, be: Optional[torch.Tensor], ce: Optional[torch.Tensor],
                  levels: List[LevelWeights], p: int, heads: int, out: Optional[torch.Tensor] = None,
                  workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """out[B,N,D]: tokenize, then every level in turn (the last must leave one group)."""
    B, C, H, W = x.shape
    D = We.shape[1]
    if tuple(We.shape) != (C, D, p * p):
        raise ValueError("We must be [C, D, p*p]")
    N = (H // p) * (W // p) if p > 0 else 0
    dt = _dt(x)
    if workspace is None:
        workspace = _workspace(dchag_workspace_bytes(dt, B, C, H, W, p, D, heads, [lv.group_size for lv in levels], 1),
                               x.device)
    if out is None:
        out = torch.empty((B, N, D), dtype=x.dtype, device=x.device)
    arr = (_CLevel * len(levels))(*[_clevel(lv, x) for lv in levels])
    _check(load_library().dchag_forward(dt, B, C, H, W, p, D, heads, _ptr(x), _ptr(We, x), _ptr(be, x), _ptr(ce, x),
                                        len(levels), arr, _ptr(out, x), ctypes.c_void_p(workspace.data_ptr()),
                                        workspace.numel(), _stream(stream)))
    return out


def dchag_forward_pos(x: torch.Tensor, We: torch.Tensor, be: Optional[torch.Tensor], ce: Optional[torch.Tensor],
                      levels: List[LevelWeights], p: int, heads: int, pos: torch.Tensor,
                      out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                      stream=None) -> torch.Tensor:
    """out[B,N,D] = dchag_forward(...) + pos[N,D], the sum taken in the last projection's epilogue."""
    B, C, H, W = x.shape
    D = We.shape[1]
    if tuple(We.shape) != (C, D, p * p):
        raise ValueError("We must be [C, D, p*p]")
    N = (H // p) * (W // p) if p > 0 else 0
    if tuple(pos.shape) != (N, D):
        raise ValueError("pos must be [N, D]")
    dt = _dt(x)
    if workspace is None:
        workspace = _workspace(dchag_workspace_bytes(dt, B, C, H, W, p, D, heads, [lv.group_size for lv in levels], 1),
                               x.device)
    if out is None:
        out = torch.empty((B, N, D), dtype=x.dtype, device=x.device)
    arr = (_CLevel * len(levels))(*[_clevel(lv, x) for lv in levels])
    _check(load_library().dchag_forward_pos(dt, B, C, H, W, p, D, heads, _ptr(x), _ptr(We, x), _ptr(be, x),
                                            _ptr(ce, x), len(levels), arr, _ptr(pos, x), _ptr(out, x),
                                            ctypes.c_void_p(workspace.data_ptr()), workspace.numel(),
                                            _stream(stream)))
    return out


def dchag_forward_folded(x: torch.Tensor, We: torch.Tensor, be: Optional[torch.Tensor], ce: Optional[torch.Tensor],
                         levels: List[LevelWeights], p: int, heads: int, out: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """out[B,N,D] as dchag_forward, with the value projection applied after the softmax-weighted sum."""
    B, C, H, W = x.shape
    D = We.shape[1]
    if tuple(We.shape) != (C, D, p * p):
        raise ValueError("We must be [C, D, p*p]")
    N = (H // p) * (W // p) if p > 0 else 0
    dt = _dt(x)
    if workspace is None:
        workspace = _workspace(dchag_workspace_bytes(dt, B, C, H, W, p, D, heads, [lv.group_size for lv in levels], 2),
                               x.device)
    if out is None:
        out = torch.empty((B, N, D), dtype=x.dtype, device=x.device)
    arr = (_CLevel * len(levels))(*[_clevel(lv, x) for lv in levels])
    _check(load_library().dchag_forward_folded(dt, B, C, H, W, p, D, heads, _ptr(x), _ptr(We, x), _ptr(be, x),
                                               _ptr(ce, x), len(levels), arr, _ptr(out, x),
                                               ctypes.c_void_p(workspace.data_ptr()), workspace.numel(),
                                               _stream(stream)))
    return out


def dchag_fold_value(We: torch.Tensor, be: Optional[torch.Tensor], ce: Optional[torch.Tensor],
                     levels: List[LevelWeights], p: int, heads: int, stream=None) -> Optional[torch.Tensor]:
    """Everything of dchag_forward_folded that depends on the weights alone, for dchag_forward_prefolded; None when
    the library does not take that shape's first level from the pixels (dchag_value_fold_bytes == 0)."""
    C, D = We.shape[0], We.shape[1]
    if tuple(We.shape) != (C, D, p * p):
        raise ValueError("We must be [C, D, p*p]")
    dt = _dt(We)
    lib = load_library()
    arr = (_CLevel * len(levels))(*[_clevel(lv, We) for lv in levels])
    need = lib.dchag_value_fold_bytes(dt, C, p, D, heads, len(levels), arr)
    if need == 0:
        return None
    folded = _workspace(need, We.device)
    _check(lib.dchag_fold_value(dt, C, p, D, heads, _ptr(We), _ptr(be, We), _ptr(ce, We), len(levels), arr,
                                ctypes.c_void_p(folded.data_ptr()), folded.numel(), _stream(stream)))
    return folded


def dchag_forward_prefolded(x: torch.Tensor, We: torch.Tensor, be: Optional[torch.Tensor], ce: Optional[torch.Tensor],
                            levels: List[LevelWeights], p: int, heads: int, folded: torch.Tensor,
                            out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                            stream=None) -> torch.Tensor:
    """dchag_forward_folded with the first level's weight-only products taken from `folded` (dchag_fold_value)."""
    B, C, H, W = x.shape
    D = We.shape[1]
    if tuple(We.shape) != (C, D, p * p):
        raise ValueError("We must be [C, D, p*p]")
    N = (H // p) * (W // p) if p > 0 else 0
    dt = _dt(x)
    if workspace is None:
        workspace = _workspace(dchag_workspace_bytes(dt, B, C, H, W, p, D, heads, [lv.group_size for lv in levels], 2),
                               x.device)
    if out is None:
        out = torch.empty((B, N, D), dtype=x.dtype, device=x.device)
    arr = (_CLevel * len(levels))(*[_clevel(lv, x) for lv in levels])
    _check(load_library().dchag_forward_prefolded(dt, B, C, H, W, p, D, heads, _ptr(x), _ptr(We, x), _ptr(be, x),
                                                  _ptr(ce, x), len(levels), arr,
                                                  ctypes.c_void_p(folded.data_ptr()), _ptr(out, x),
                                                  ctypes.c_void_p(workspace.data_ptr()), workspace.numel(),
                                                  _stream(stream)))
    return out


def dchag_forward_keep(x: torch.Tensor, We: torch.Tensor, be: Optional[torch.Tensor], ce: Optional[torch.Tensor],
                       levels: List[LevelWeights], p: int, heads: int, workspace: torch.Tensor,
                       out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """out[B,N,D] as dchag_forward_folded; `workspace` (dchag_workspace_bytes(..., 3) bytes) keeps what
    dchag_backward_kept reads."""
    B, C, H, W = x.shape
    D = We.shape[1]
    if tuple(We.shape) != (C, D, p * p):
        raise ValueError("We must be [C, D, p*p]")
    N = (H // p) * (W // p) if p > 0 else 0
    if out is None:
        out = torch.empty((B, N, D), dtype=x.dtype, device=x.device)
    arr = (_CLevel * len(levels))(*[_clevel(lv, x) for lv in levels])
    _check(load_library().dchag_forward_keep(_dt(x), B, C, H, W, p, D, heads, _ptr(x), _ptr(We, x), _ptr(be, x),
                                             _ptr(ce, x), len(levels), arr, _ptr(out, x),
                                             ctypes.c_void_p(workspace.data_ptr()), workspace.numel(), _stream(stream)))
    return out


def dchag_backward(x: torch.Tensor, We: torch.Tensor, be: Optional[torch.Tensor], ce: Optional[torch.Tensor],
                   levels: List[LevelWeights], p: int, heads: int, dout: torch.Tensor,
                   grads: List[LevelGrads], dx: Optional[torch.Tensor] = None, dWe: Optional[torch.Tensor] = None,
                   dtok_bias: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                   stream=None, kept: bool = False) -> None:
    """Writes the gradients of <dout, dchag_forward(...)> into the given tensors (None = not wanted).
    kept=True calls dchag_backward_kept: `workspace` must be the one a dchag_forward_keep call just filled."""
    B, C, H, W = x.shape
    D = We.shape[1]
    if tuple(We.shape) != (C, D, p * p):
        raise ValueError("We must be [C, D, p*p]")
    if len(grads) != len(levels):
        raise ValueError("one LevelGrads per level")
    dt = _dt(x)
    if workspace is None:
        workspace = _workspace(dchag_workspace_bytes(dt, B, C, H, W, p, D, heads, [lv.group_size for lv in levels], 3),
                               x.device)
    arr = (_CLevel * len(levels))(*[_clevel(lv, x) for lv in levels])
    garr = (_CLevelGrads * len(levels))()
    for j, g in enumerate(grads):
        for name in ("dquery", "dWq", "dWk", "dWv", "dWo", "dbq", "dbk", "dbv", "dbo"):
            setattr(garr[j], name, _ptr(getattr(g, name), x))
    if kept and workspace is None:
        raise ValueError("kept=True needs the workspace of the dchag_forward_keep call")
    fn = load_library().dchag_backward_kept if kept else load_library().dchag_backward
    _check(fn(dt, B, C, H, W, p, D, heads, _ptr(x), _ptr(We, x), _ptr(be, x), _ptr(ce, x),
              len(levels), arr, _ptr(dout, x), _ptr(dx, x), _ptr(dWe, x), _ptr(dtok_bias, x), garr,
              ctypes.c_void_p(workspace.data_ptr()), workspace.numel(), _stream(stream)))


def dchag_yardstick_mfma(iters: int, sink: torch.Tensor, stream=None) -> float:
    """Launches the MFMA-only yardstick loop; returns the flops it performs.  sink: float32 device scratch."""
    flops = ctypes.c_double(0.0)
    _check(load_library().dchag_yardstick_mfma(int(iters), ctypes.c_void_p(sink.data_ptr()), sink.numel(),
                                               ctypes.byref(flops), _stream(stream)))
    return float(flops.value)


def dchag_yardstick_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> int:
    """Launches the stream-copy yardstick dst <- src; returns the bytes read (= the bytes written)."""
    nbytes = src.numel() * src.element_size()
    _check(load_library().dchag_yardstick_copy(ctypes.c_void_p(dst.data_ptr()), ctypes.c_void_p(src.data_ptr()),
                                               nbytes, _stream(stream)))
    return nbytes


def dchag_yardstick_read(src: torch.Tensor, sink: torch.Tensor, stream=None) -> int:
    """Launches the streaming-read yardstick over src; returns the bytes read.  sink: float32 device scratch (>= 256)."""
    nbytes = src.numel() * src.element_size()
    _check(load_library().dchag_yardstick_read(ctypes.c_void_p(src.data_ptr()), nbytes,
                                               ctypes.c_void_p(sink.data_ptr()), _stream(stream)))
    return nbytes


def dchag_profile_begin() -> None:
    """Start bracketing every kernel launch of the library with HIP events (benchmark diagnostic)."""
    _check(load_library().dchag_profile_begin())


def dchag_profile_end(cap: int = 1 << 16):
    """Stop stage timing; returns [(stage name, level, ms)] in launch order."""
    buf = (_CStageTime * cap)()
    n = load_library().dchag_profile_end(buf, cap)
    if n < 0:
        _check(n)
    return [(STAGE_NAMES.get(buf[j].stage, str(buf[j].stage)), int(buf[j].level), float(buf[j].ms))
            for j in range(min(n, cap))]
