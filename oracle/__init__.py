"""ctypes front end of the fp64 CPU oracle (``dchag_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this package.  It imports nothing of the GPU library and the GPU library
imports nothing of it.

All functions take float32 numpy arrays for inputs and weights (bf16 values are
exactly representable in float32) and return float64 arrays.  A "level" is any
object with the attributes ``group_size, query, Wq, Wk, Wv, Wo, bq, bk, bv, bo``
(biases may be None) and optionally ``kind`` ("attention", the default, or "linear":
then ``Wv`` holds the channel-mixing weights [G, g, D], ``bv`` the bias [G, D], and
the other arrays are ignored).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dchag_oracle.c")
_LIB_PATH = os.path.join(_HERE, "libdchag_oracle.so")

_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_i32p = ctypes.POINTER(ctypes.c_int32)


class _CLevel(ctypes.Structure):
    _fields_ = [("group_size", ctypes.c_int32), ("kind", ctypes.c_int32),
                ("query", _f32p),
                ("Wq", _f32p), ("Wk", _f32p), ("Wv", _f32p), ("Wo", _f32p),
                ("bq", _f32p), ("bk", _f32p), ("bv", _f32p), ("bo", _f32p)]


class _CLevelGrad(ctypes.Structure):
    _fields_ = [("dquery", _f64p),
                ("dWq", _f64p), ("dWk", _f64p), ("dWv", _f64p), ("dWo", _f64p),
                ("dbq", _f64p), ("dbk", _f64p), ("dbv", _f64p), ("dbo", _f64p)]


def compile_source(src: str, lib_path: str) -> str:
    """gcc line used for the oracle: OpenMP, -O2, no fast-math (fp64 sums stay in source order)."""
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", lib_path, src, "-lm"]
    subprocess.run(cmd, check=True)
    return lib_path


def build(force: bool = False) -> str:
    """Compile the oracle into a shared library beside its source (if missing or out of date)."""
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(_SRC):
        compile_source(_SRC, _LIB_PATH)
    return _LIB_PATH


_libs = {}


def use_library(path: Optional[str]) -> None:
    """Point the front end at another build of the oracle (tests of the pins use a
    deliberately broken copy); None restores the default library."""
    global _active
    _active = path


_active: Optional[str] = None


def _load():
    path = _active or _LIB_PATH
    if path not in _libs:
        if path == _LIB_PATH:
            build()
        lib = ctypes.CDLL(path)
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_threads.argtypes = [ctypes.c_int]
        lib.oracle_tokenize.restype = ctypes.c_int
        lib.oracle_tokenize.argtypes = [ctypes.c_int] * 6 + [_f32p] * 4 + [ctypes.c_int, _i32p, _i32p, _f64p]
        lib.oracle_aggregate_level.restype = ctypes.c_int
        lib.oracle_aggregate_level.argtypes = [ctypes.c_int] * 4 + [ctypes.POINTER(_CLevel), _f64p, _f64p, _f64p, _f64p]
        lib.oracle_forward.restype = ctypes.c_int
        lib.oracle_forward.argtypes = ([ctypes.c_int] * 7 + [_f32p] * 4 + [ctypes.c_int, ctypes.POINTER(_CLevel)]
                                       + [ctypes.c_int, _i32p, _i32p, _f64p])
        lib.oracle_add_positional.restype = ctypes.c_int
        lib.oracle_add_positional.argtypes = [ctypes.c_int] * 3 + [_i32p, _f32p, _f64p]
        lib.oracle_backward.restype = ctypes.c_int
        lib.oracle_backward.argtypes = ([ctypes.c_int] * 7 + [_f32p] * 4 + [ctypes.c_int, ctypes.POINTER(_CLevel)]
                                        + [ctypes.c_int, _i32p, _i32p, _f64p, _f64p, _f64p, _f64p,
                                           ctypes.POINTER(_CLevelGrad)])
        _libs[path] = lib
    return _libs[path]


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_threads(n: int) -> None:
    _load().oracle_set_threads(int(n))


def _f32(a, shape=None, keep=None):
    if a is None:
        return None, None
    arr = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None and tuple(arr.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(arr.shape)}")
    if keep is not None:
        keep.append(arr)
    return arr, arr.ctypes.data_as(_f32p)


def _clevel(lv, c_in: int, D: int, keep: list) -> _CLevel:
    g = int(lv.group_size)
    G = (c_in + g - 1) // g
    c = _CLevel()
    c.group_size = g
    if getattr(lv, "kind", "attention") == "linear":
        c.kind = 1
        c.Wv = _f32(lv.Wv, (G, g, D), keep)[1]
        c.bv = _f32(lv.bv, (G, D), keep)[1]
        return c
    c.kind = 0
    c.query = _f32(lv.query, (G, D), keep)[1]
    for name in ("Wq", "Wk", "Wv", "Wo"):
        setattr(c, name, _f32(getattr(lv, name), (G, D, D), keep)[1])
    for name in ("bq", "bk", "bv", "bo"):
        setattr(c, name, _f32(getattr(lv, name), (G, D), keep)[1])
    return c


def _samples(B: int, N: int, sample):
    if sample is None:
        sb = np.repeat(np.arange(B, dtype=np.int32), N)
        sn = np.tile(np.arange(N, dtype=np.int32), B)
    else:
        sb = np.ascontiguousarray(sample[0], dtype=np.int32)
        sn = np.ascontiguousarray(sample[1], dtype=np.int32)
        if sb.shape != sn.shape or sb.ndim != 1:
            raise ValueError("sample must be two 1-D arrays of equal length")
    return sb, sn


def tokenize(x, We, be, ce, p: int, sample=None) -> np.ndarray:
    """Tokens of the sampled patches, float64 [S, C, D]; with sample=None, S = B*N in (b, n) order."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    B, C, H, W = x.shape
    We = np.ascontiguousarray(We, dtype=np.float32)
    D = We.shape[1]
    if We.shape != (C, D, p * p):
        raise ValueError("We must be [C, D, p*p]")
    N = (H // p) * (W // p)
    sb, sn = _samples(B, N, sample)
    keep: list = []
    out = np.empty((sb.size, C, D), dtype=np.float64)
    rc = _load().oracle_tokenize(B, C, H, W, p, D, x.ctypes.data_as(_f32p), We.ctypes.data_as(_f32p),
                                 _f32(be, (C, D), keep)[1], _f32(ce, (C, D), keep)[1], sb.size,
                                 sb.ctypes.data_as(_i32p), sn.ctypes.data_as(_i32p), out.ctypes.data_as(_f64p))
    if rc != 0:
        raise ValueError(f"oracle_tokenize rejected the shape (rc={rc})")
    return out


def aggregate_level(z, lv, heads: int, want_alpha: bool = False, want_pre: bool = False):
    """One level on independent patches: z float64 [S, c_in, D] -> y float64 [S, G, D].

    With want_alpha / want_pre also returns the softmax weights [S, c_in, heads]
    and the concatenated heads before the output projection [S, G, D].
    """
    z = np.ascontiguousarray(z, dtype=np.float64)
    S, c_in, D = z.shape
    keep: list = []
    cl = _clevel(lv, c_in, D, keep)
    G = (c_in + cl.group_size - 1) // cl.group_size
    y = np.empty((S, G, D), dtype=np.float64)
    alpha = np.empty((S, c_in, heads), dtype=np.float64) if want_alpha else None
    pre = np.empty((S, G, D), dtype=np.float64) if want_pre else None
    rc = _load().oracle_aggregate_level(S, c_in, D, heads, ctypes.byref(cl), z.ctypes.data_as(_f64p),
                                        y.ctypes.data_as(_f64p),
                                        alpha.ctypes.data_as(_f64p) if want_alpha else None,
                                        pre.ctypes.data_as(_f64p) if want_pre else None)
    if rc != 0:
        raise ValueError(f"oracle_aggregate_level rejected the shape (rc={rc})")
    res = (y,)
    if want_alpha:
        res += (alpha,)
    if want_pre:
        res += (pre,)
    return res[0] if len(res) == 1 else res


def forward(x, We, be, ce, levels: Sequence, p: int, heads: int, sample=None, pos=None) -> np.ndarray:
    """The whole path on the sampled patches: float64 [S, D] (S = B*N in (b, n) order if sample is None);
    with pos [N, D] the positional embedding of each patch is added to its output."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    B, C, H, W = x.shape
    We = np.ascontiguousarray(We, dtype=np.float32)
    D = We.shape[1]
    if We.shape != (C, D, p * p):
        raise ValueError("We must be [C, D, p*p]")
    N = (H // p) * (W // p)
    sb, sn = _samples(B, N, sample)
    keep: list = []
    arr = (_CLevel * len(levels))()
    c_in = C
    for i, lv in enumerate(levels):
        arr[i] = _clevel(lv, c_in, D, keep)
        c_in = (c_in + arr[i].group_size - 1) // arr[i].group_size
    out = np.empty((sb.size, D), dtype=np.float64)
    rc = _load().oracle_forward(B, C, H, W, p, D, heads, x.ctypes.data_as(_f32p), We.ctypes.data_as(_f32p),
                                _f32(be, (C, D), keep)[1], _f32(ce, (C, D), keep)[1], len(levels), arr,
                                sb.size, sb.ctypes.data_as(_i32p), sn.ctypes.data_as(_i32p),
                                out.ctypes.data_as(_f64p))
    if rc != 0:
        raise ValueError(f"oracle_forward rejected the shape (rc={rc})")
    if pos is not None:
        pa, pp_ = _f32(pos, (N, D), keep)
        rc = _load().oracle_add_positional(N, D, sb.size, sn.ctypes.data_as(_i32p), pp_, out.ctypes.data_as(_f64p))
        if rc != 0:
            raise ValueError(f"oracle_add_positional rejected the sample (rc={rc})")
    return out


def backward(x, We, be, ce, levels: Sequence, p: int, heads: int, dout, sample=None, want_dx: bool = True) -> dict:
    """Gradients of L = sum_i <dout[i], out[i]> over the sampled patches (all B*N patches in (b, n)
    order if sample is None); dout is [S, D].

    Returns {"dx": [S, C, p*p] or None (pixel gradients of each sampled patch, row by row),
    "dWe": [C, D, p*p], "dtok_bias": [C, D] (the gradient of be and of ce alike),
    "levels": [{"dquery", "dWq", "dWk", "dWv", "dWo", "dbq", "dbk", "dbv", "dbo"}, ...]}, all float64;
    a linear level has only "dWv" [G, g, D] and "dbv".
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    B, C, H, W = x.shape
    We = np.ascontiguousarray(We, dtype=np.float32)
    D = We.shape[1]
    if We.shape != (C, D, p * p):
        raise ValueError("We must be [C, D, p*p]")
    N = (H // p) * (W // p)
    sb, sn = _samples(B, N, sample)
    dout = np.ascontiguousarray(dout, dtype=np.float64)
    if dout.shape != (sb.size, D):
        raise ValueError("dout must be [S, D]")
    keep: list = []
    arr = (_CLevel * len(levels))()
    garr = (_CLevelGrad * len(levels))()
    res_levels = []
    c_in = C
    for i, lv in enumerate(levels):
        arr[i] = _clevel(lv, c_in, D, keep)
        g = arr[i].group_size
        G = (c_in + g - 1) // g
        d = {}
        if arr[i].kind == 1:
            d["dWv"] = np.zeros((G, g, D))
            d["dbv"] = np.zeros((G, D))
        else:
            d["dquery"] = np.zeros((G, D))
            for name in ("dWq", "dWk", "dWv", "dWo"):
                d[name] = np.zeros((G, D, D))
            for name in ("dbq", "dbk", "dbv", "dbo"):
                d[name] = np.zeros((G, D))
        for name, a in d.items():
            setattr(garr[i], name, a.ctypes.data_as(_f64p))
        res_levels.append(d)
        c_in = G
    dx = np.zeros((sb.size, C, p * p)) if want_dx else None
    dWe = np.zeros((C, D, p * p))
    dtb = np.zeros((C, D))
    rc = _load().oracle_backward(B, C, H, W, p, D, heads, x.ctypes.data_as(_f32p), We.ctypes.data_as(_f32p),
                                 _f32(be, (C, D), keep)[1], _f32(ce, (C, D), keep)[1], len(levels), arr,
                                 sb.size, sb.ctypes.data_as(_i32p), sn.ctypes.data_as(_i32p),
                                 dout.ctypes.data_as(_f64p), dx.ctypes.data_as(_f64p) if want_dx else None,
                                 dWe.ctypes.data_as(_f64p), dtb.ctypes.data_as(_f64p), garr)
    if rc != 0:
        raise ValueError(f"oracle_backward rejected the shape (rc={rc})")
    return {"dx": dx, "dWe": dWe, "dtok_bias": dtb, "levels": res_levels}
