"""dchag_aggregate_level_static (the entry point that allocates nothing: its workspace is a fixed array inside the
library) against dchag_aggregate_level on a caller-owned workspace, through the C ABI.

The two calls run the same kernels on the same workspace layout, so their outputs must be equal bit for bit.  Two
calls in a row share the array: the second, smaller one must not be disturbed by what the first left behind.
This file is collected last (its name sorts after every other test file) on purpose.
"""
import ctypes
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2506_21411_amd as dchag
from paper_2506_21411_amd.binding import _clevel
from workloads import make_level, make_tokens

pytestmark = pytest.mark.gpu

TDT = {"f32": torch.float32, "bf16": torch.bfloat16}


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def problem(dtype, B, Cin, N, D, heads, g, seed):
    """Seeded tokens and one attention level, on the host (oracle input) and on the device."""
    G = (Cin + g - 1) // g
    z = make_tokens(B, Cin, N, D, dtype, seed)
    lv = make_level(np.random.Generator(np.random.PCG64(seed + 100)), G, g, D, dtype, True)

    def dev(a):
        return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to("cuda").to(TDT[dtype]).contiguous()

    dlv = dchag.LevelWeights(lv.group_size, dev(lv.query), dev(lv.Wq), dev(lv.Wk), dev(lv.Wv), dev(lv.Wo),
                             dev(lv.bq), dev(lv.bk), dev(lv.bv), dev(lv.bo))
    return z, lv, dev(z), dlv


def both_ways(dtype, B, Cin, N, D, heads, g, seed):
    z, lv, dz, dlv = problem(dtype, B, Cin, N, D, heads, g, seed)
    G = (Cin + g - 1) // g
    say(f"static-scratch level: {dtype} B={B} Cin={Cin} N={N} D={D} heads={heads} g={g}")
    want = dchag.dchag_aggregate_level(dz, dlv, heads)
    got = torch.full((B, G, N, D), float("nan"), dtype=TDT[dtype], device="cuda")
    dchag.dchag_aggregate_level_static(dz, dlv, heads, got)
    torch.cuda.synchronize()
    assert torch.equal(got, want), "static-scratch call differs from the workspace call"
    # and both against the oracle, to the tolerance of the parity tests
    zo = z.transpose(0, 2, 1, 3).reshape(B * N, Cin, D)
    ref = oracle.aggregate_level(zo, lv, heads).reshape(B, N, -1, D).transpose(0, 2, 1, 3)
    err = float(np.abs(got.to(torch.float64).cpu().numpy() - ref).max() / np.abs(ref).max())
    say(f"  max|err|/max|ref| against the oracle = {err:.3e}")
    assert err < (1e-4 if dtype == "f32" else 2e-2)


def test_two_calls_in_a_row_second_smaller():
    # bf16 MFMA path: 3 groups (last short), 2 patch tiles with a ragged tail; needs about 1.5 MiB of scratch
    both_ways("bf16", 2, 20, 40, 256, 4, 8, seed=11)
    # smaller on every axis, so it uses a prefix of what the first call wrote
    both_ways("bf16", 1, 5, 17, 256, 4, 3, seed=12)
    # the fp32 (shape-generic) kernels on the same array
    both_ways("f32", 1, 8, 24, 64, 4, 4, seed=13)
    both_ways("f32", 1, 3, 5, 32, 2, 2, seed=14)


def test_oversized_level_is_rejected_before_any_launch():
    lib = dchag.load_library()
    need = dchag.dchag_workspace_bytes(dchag.DCHAG_BF16, 4, 512, 256, 1, 1, 1024, 16, [32], 0)
    assert need > dchag.STATIC_SCRATCH_BYTES           # the headline level needs more than the fixed array holds
    z, lv, dz, dlv = problem("bf16", 1, 4, 8, 256, 4, 4, seed=15)
    cl = _clevel(dlv, dz)
    sentinel = torch.full((8,), 7.0, dtype=torch.bfloat16, device="cuda")
    # shapes of the headline level with pointers of a small problem: validation fails on the size, nothing is launched
    rc = lib.dchag_aggregate_level_static(dchag.DCHAG_BF16, 4, 512, 256, 1024, 16, ctypes.byref(cl),
                                          ctypes.c_void_p(dz.data_ptr()), ctypes.c_void_p(sentinel.data_ptr()), None)
    torch.cuda.synchronize()
    assert rc == -4
    assert bool((sentinel == 7.0).all())
