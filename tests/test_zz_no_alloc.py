"""liec_l2_norm_static, the entry point for callers that cannot allocate: its output against
liec_l2_norm's on two calls in a row, the second with a smaller input, through the C ABI."""
import ctypes
import math
import os
import sys

import numpy as np
import pytest
import torch

sys.path.insert(0, os.path.dirname(__file__))
from _gpu import DEV, GPU_MARKS, say  # noqa: E402

pytestmark = GPU_MARKS

# fp64 sums of the same squares in two fixed orders: a few units in the last place apart
REL_TOL = 1e-13


def _both(lib, ctx, vec, n, out):
    want = ctypes.c_double()
    assert lib.liec_l2_norm(ctx, vec.data_ptr(), n, ctypes.byref(want)) == 0
    stream = torch.cuda.current_stream().cuda_stream
    assert lib.liec_l2_norm_static(vec.data_ptr(), n, out.data_ptr(), stream) == 0
    torch.cuda.synchronize()
    return float(out.cpu()[0]), float(want.value)


def test_static_l2_norm_matches_the_allocating_one_on_two_calls_in_a_row():
    import paper_2402_11857_amd as pkg

    lib = pkg.lib()
    say("case no-alloc entry point: liec_l2_norm_static against liec_l2_norm, n = 3 000 001 then 70 001")
    gen = torch.Generator(device=DEV)
    gen.manual_seed(5)
    vec = torch.randn(3_000_001, generator=gen, device=DEV, dtype=torch.float32) * 3.0
    out = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
    h = ctypes.c_void_p()
    assert lib.liec_create(ctypes.byref(h), 2, 4096, 1, 0, 0.1) == 0
    try:
        for n in (3_000_001, 70_001):                 # the second call reuses the array the first one filled
            got, want = _both(lib, h, vec, n, out)
            ref = math.sqrt(float(np.sum(vec[:n].cpu().numpy().astype(np.float64) ** 2)))
            assert abs(got - want) <= REL_TOL * want, f"n={n}: static {got!r} against allocating {want!r}"
            assert abs(got - ref) <= 1e-12 * ref, f"n={n}: static {got!r} against the host sum {ref!r}"
        # one value, and a vector of zeros
        got, want = _both(lib, h, vec, 1, out)
        assert got == want == abs(float(vec[0]))
        zeros = torch.zeros(1000, dtype=torch.float32, device=DEV)
        got, want = _both(lib, h, zeros, 1000, out)
        assert got == want == 0.0
    finally:
        lib.liec_destroy(h)


def test_static_l2_norm_rejects_what_it_cannot_take():
    import paper_2402_11857_amd as pkg

    lib = pkg.lib()
    say("case no-alloc entry point: argument checks")
    vec = torch.ones(16, dtype=torch.float32, device=DEV)
    out = torch.zeros(2, dtype=torch.float64, device=DEV)
    assert lib.liec_l2_norm_static(None, 16, out.data_ptr(), None) == 1
    assert lib.liec_l2_norm_static(vec.data_ptr(), 16, None, None) == 1
    assert lib.liec_l2_norm_static(vec.data_ptr(), 0, out.data_ptr(), None) == 1
    assert lib.liec_l2_norm_static(vec.data_ptr(), (1 << 32) + 1, out.data_ptr(), None) == 1     # beyond the maximum
    assert lib.liec_l2_norm_static(vec.data_ptr() + 2, 8, out.data_ptr(), None) == 1             # misaligned input
    assert lib.liec_l2_norm_static(vec.data_ptr(), 16, out.data_ptr() + 4, None) == 1            # misaligned output
    torch.cuda.synchronize()
    assert float(out.cpu()[0]) == 0.0                 # nothing ran
    pkg.liec_l2_norm_static(vec, out)
    torch.cuda.synchronize()
    assert float(out.cpu()[0]) == 4.0
