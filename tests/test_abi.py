"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
include/dchag.h declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

import paper_2506_21411_amd as dchag
from paper_2506_21411_amd.binding import _CLevel

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000          # never dereferenced: every call below fails validation first


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(dchag.library_path()):
        from paper_2506_21411_amd.build import build
        build(verbose=False)
    return dchag.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "dchag.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dchag_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"dchag_tokenize", "dchag_aggregate_level", "dchag_forward", "dchag_workspace_bytes",
            "dchag_strerror", "dchag_version", "dchag_forward_folded", "dchag_backward",
            "dchag_forward_pos", "dchag_forward_keep", "dchag_backward_kept"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in dchag.h but not exported"


def test_strerror_and_version(lib):
    assert lib.dchag_version().decode().count(".") == 1
    for s in range(-6, 1):
        assert lib.dchag_strerror(s)
    assert lib.dchag_strerror(-99) == b"unknown status"


def level(g=4, **over):
    c = _CLevel()
    c.group_size, c.kind = g, 0
    for n in ("query", "Wq", "Wk", "Wv", "Wo"):
        setattr(c, n, FAKE)
    for k, v in over.items():
        setattr(c, k, v)
    return c


def test_tokenize_validation(lib):
    t = lib.dchag_tokenize
    assert t(0, 1, 8, 32, 64, 4, 128, None, FAKE, None, None, FAKE, None) == -1
    assert t(0, 1, 8, 32, 64, 4, 128, FAKE, FAKE, None, None, None, None) == -1
    assert t(0, 1, 8, 30, 64, 4, 128, FAKE, FAKE, None, None, FAKE, None) == -2      # H % p
    assert t(0, 1, 8, 32, 62, 4, 128, FAKE, FAKE, None, None, FAKE, None) == -2      # W % p
    assert t(0, 1, 8, 32, 64, 4, 124, FAKE, FAKE, None, None, FAKE, None) == -2      # D % 8
    assert t(0, 0, 8, 32, 64, 4, 128, FAKE, FAKE, None, None, FAKE, None) == -2      # B < 1
    assert t(7, 1, 8, 32, 64, 4, 128, FAKE, FAKE, None, None, FAKE, None) == -3      # dtype
    assert t(0, 1, 8, 32, 64, 4, 128, FAKE + 4, FAKE, None, None, FAKE, None) == -6  # alignment


def test_aggregate_level_validation(lib):
    a = lib.dchag_aggregate_level
    lv = level(4)
    assert a(0, 1, 8, 128, 128, 4, None, FAKE, FAKE, FAKE, 1 << 30, None) == -1
    assert a(0, 1, 8, 128, 128, 4, ctypes.byref(lv), None, FAKE, FAKE, 1 << 30, None) == -1
    assert a(0, 1, 8, 128, 128, 3, ctypes.byref(lv), FAKE, FAKE, FAKE, 1 << 30, None) == -2   # D % heads
    assert a(0, 1, 8, 128, 128, 4, ctypes.byref(level(0)), FAKE, FAKE, FAKE, 1 << 30, None) == -2
    assert a(0, 1, 8, 128, 128, 4, ctypes.byref(level(4, Wv=None)), FAKE, FAKE, FAKE, 1 << 30, None) == -1
    assert a(0, 1, 8, 128, 128, 4, ctypes.byref(lv), FAKE, FAKE, None, 1 << 30, None) == -4
    assert a(0, 1, 8, 128, 128, 4, ctypes.byref(lv), FAKE, FAKE, FAKE, 16, None) == -4          # too small
    assert a(0, 1, 8, 128, 128, 4, ctypes.byref(lv), FAKE, FAKE, FAKE + 16, 1 << 30, None) == -4  # misaligned


def test_aggregate_level_static_validation(lib):
    """The entry point without a workspace argument: same checks, and a level that does not fit the library's fixed
    scratch array is turned down on the host (no GPU is needed to find that out)."""
    a = lib.dchag_aggregate_level_static
    lv = level(4)
    assert a(0, 1, 8, 128, 128, 4, None, FAKE, FAKE, None) == -1
    assert a(0, 1, 8, 128, 128, 4, ctypes.byref(lv), None, FAKE, None) == -1
    assert a(0, 1, 8, 128, 128, 3, ctypes.byref(lv), FAKE, FAKE, None) == -2                  # D % heads
    assert a(7, 1, 8, 128, 128, 4, ctypes.byref(lv), FAKE, FAKE, None) == -3
    big = level(32)
    assert dchag.dchag_workspace_bytes(dchag.DCHAG_BF16, 4, 512, 256, 1, 1, 1024, 16, [32], 0) > dchag.STATIC_SCRATCH_BYTES
    assert a(1, 4, 512, 256, 1024, 16, ctypes.byref(big), FAKE, FAKE, None) == -4              # needs more than 32 MiB


def test_yardstick_validation(lib):
    """The benchmark's yardstick calls check their arguments on the host like every other entry point."""
    flops = ctypes.c_double(0.0)
    ym = lib.dchag_yardstick_mfma
    ym.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
    assert ym(10, None, 1 << 30, ctypes.byref(flops), None) == -1
    assert ym(0, FAKE, 1 << 30, ctypes.byref(flops), None) == -2
    assert ym(10, FAKE, 16, ctypes.byref(flops), None) == -4                     # scratch too small
    yc = lib.dchag_yardstick_copy
    yc.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    assert yc(None, FAKE, 1024, None) == -1
    assert yc(FAKE, FAKE, 1000, None) == -2                                      # not a multiple of 16 bytes
    assert yc(FAKE + 4, FAKE, 1024, None) == -6
    yr = lib.dchag_yardstick_read
    yr.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
    assert yr(FAKE, 1024, None, None) == -1
    assert yr(FAKE, 0, FAKE, None) == -2


def test_forward_validation(lib):
    f = lib.dchag_forward
    two = (_CLevel * 2)(level(4), level(2))
    bad_chain = (_CLevel * 2)(level(4), level(1))        # leaves two groups
    args = lambda lv, n, ws=FAKE, wsb=1 << 40: (0, 1, 8, 32, 64, 4, 128, 4, FAKE, FAKE, None, None, n, lv,
                                                 FAKE, ws, wsb, None)
    assert f(*args(two, 0)) == -2
    assert f(*args(bad_chain, 2)) == -2
    assert f(*args(two, 2, wsb=1024)) == -4
    assert f(*args(two, 2, ws=None)) == -4
    assert f(*args(None, 2)) == -1


def test_forward_folded_and_backward_validation(lib):
    from paper_2506_21411_amd.binding import _CLevelGrads
    two = (_CLevel * 2)(level(4), level(2))
    bad_chain = (_CLevel * 2)(level(4), level(1))
    ff = lib.dchag_forward_folded
    args = lambda lv, n, ws=FAKE, wsb=1 << 40: (0, 1, 8, 32, 64, 4, 128, 4, FAKE, FAKE, None, None, n, lv,
                                                 FAKE, ws, wsb, None)
    assert ff(*args(two, 0)) == -2
    assert ff(*args(bad_chain, 2)) == -2
    assert ff(*args(two, 2, wsb=1024)) == -4
    assert ff(*args(None, 2)) == -1
    bw = lib.dchag_backward
    gr = (_CLevelGrads * 2)()
    bargs = lambda lv, n, dout=FAKE, g=gr, ws=FAKE, wsb=1 << 40: (0, 1, 8, 32, 64, 4, 128, 4, FAKE, FAKE, None, None, n,
                                                                   lv, dout, None, None, None, g, ws, wsb, None)
    assert bw(*bargs(two, 2, dout=None)) == -1
    assert bw(*bargs(two, 2, g=None)) == -1
    assert bw(*bargs(bad_chain, 2)) == -2
    assert bw(*bargs(two, 2, wsb=4096)) == -4
    assert bw(*bargs(two, 2, ws=None)) == -4
    gr[1].dWv = FAKE + 2
    assert bw(*bargs(two, 2)) == -6                                                     # misaligned gradient
    gr[1].dWv = FAKE
    bk, fk = lib.dchag_backward_kept, lib.dchag_forward_keep
    assert bk(*bargs(two, 2, dout=None)) == -1
    assert bk(*bargs(two, 2, wsb=4096)) == -4
    assert fk(*args(two, 2, wsb=4096)) == -4
    assert fk(0, 1, 8, 32, 64, 4, 128, 4, FAKE, FAKE, None, None, 2, two, None, FAKE, 1 << 40, None) == -1   # out


def test_forward_pos_validation(lib):
    two = (_CLevel * 2)(level(4), level(2))
    f = lib.dchag_forward_pos
    args = lambda pos, out=FAKE: (0, 1, 8, 32, 64, 4, 128, 4, FAKE, FAKE, None, None, 2, two, pos, out, FAKE, 1 << 40,
                                  None)
    assert f(*args(None)) == -1                       # the positional embedding is required by this call
    assert f(*args(FAKE + 2)) == -6
    assert f(*args(FAKE, out=None)) == -1


def test_workspace_bytes(lib):
    w0 = dchag.dchag_workspace_bytes(dchag.DCHAG_F32, 1, 8, 128, 1, 1, 128, 4, [4], 0)
    w1 = dchag.dchag_workspace_bytes(dchag.DCHAG_F32, 1, 8, 32, 64, 4, 128, 4, [4, 2], 1)
    assert w0 > 0 and w1 > w0 and w0 % 256 == 0 and w1 % 256 == 0
    assert dchag.dchag_workspace_bytes(dchag.DCHAG_F32, 1, 8, 32, 64, 4, 128, 4, [4, 1], 1) == 0   # bad chain
    assert dchag.dchag_workspace_bytes(5, 1, 8, 32, 64, 4, 128, 4, [4, 2], 1) == 0
    w2 = dchag.dchag_workspace_bytes(dchag.DCHAG_F32, 1, 8, 32, 64, 4, 128, 4, [4, 2], 2)
    w3 = dchag.dchag_workspace_bytes(dchag.DCHAG_F32, 1, 8, 32, 64, 4, 128, 4, [4, 2], 3)
    assert w2 > 0 and w3 > w2 and w2 % 256 == 0 and w3 % 256 == 0
    assert dchag.dchag_workspace_bytes(dchag.DCHAG_F32, 1, 8, 32, 64, 4, 128, 4, [4, 1], 3) == 0
    # bf16 tensors are half the size of fp32 ones
    b = dchag.dchag_workspace_bytes(dchag.DCHAG_BF16, 4, 512, 128, 128, 8, 1024, 16, [32, 16], 1)
    assert b >= 4 * 512 * 256 * 1024 * 2
