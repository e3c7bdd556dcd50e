"""The allocation-free column-sum entry point (mp_colsum_static: partial sums in a fixed array inside the library's
device image) against mp_colsum with a caller workspace, through the C ABI: same kernels and summation order, so the
same bits, and both equal the oracle.  Two calls in a row, the second with a smaller input (the array keeps the first
call's partial sums), then a shape beyond the built-in limit."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_1805_10387_amd as mp
from paper_1805_10387_amd import _lib as ML
from oracle import MIXED
from oracle.numerics import half_bits
from gpu_util import *


def _one(rows, cols, ld, seed, st=None):
    r = np.random.default_rng(seed)
    dy = MIXED.store(r.standard_normal((rows, ld)))
    ref = MIXED.store(dy[:, :cols].sum(0, dtype=np.float32))
    dyd = h16(dy)
    a = torch.full((cols,), 7.0, dtype=torch.float16, device="cuda")
    b = torch.full((cols,), 9.0, dtype=torch.float16, device="cuda")
    mp.mp_colsum(rows, cols, dyd, ld, a, None, ws_bytes(mp.mp_colsum_workspace_bytes(rows, cols)))
    free0 = torch.cuda.memory_allocated()
    mp.mp_colsum_static(rows, cols, dyd, ld, b, st)
    assert torch.cuda.memory_allocated() == free0
    torch.cuda.synchronize()
    assert np.array_equal(bits(a), bits(b)), f"{rows}x{cols}: static entry point differs from mp_colsum"
    assert_close16(b, ref, 1e-3, max_ulp=1, what=f"colsum static {rows}x{cols}")


def test_colsum_static_matches_workspace_entry_point_on_consecutive_calls():
    assert mp.mp_colsum_static_max_bytes() == 1 << 20
    _one(8192, 4096, 4096, 1)            # the bias gradient of config 3's feed-forward layer: 16 row blocks x 4096 partials
    _one(777, 1000, 1000, 2)             # smaller, right behind it: the array still holds the first call's partial sums
    _one(8192, 4096, 4096, 1)
    _one(100, 40, 48, 3)                 # leading dimension wider than the row
    _one(33, 37, 37, 4)                  # scalar path
    _one(1, 8, 8, 5)
    _one(4096, 32768, 32768, 6)          # config 4's vocabulary bias


def test_colsum_static_flags_overflow_and_rejects_what_does_not_fit():
    st = mp.scale_state_alloc()
    mp.mp_scale_state_init(st, ML.MP_SCALE_BACKOFF, 2.0 ** 15, 10)
    rows, cols = 4096, 256
    dy = np.full((rows, cols), 1.0, np.float32)
    dy[:, 17] = 100.0
    db = empty16(cols)
    mp.mp_colsum_static(rows, cols, h16(dy), cols, db, st)
    assert mp.scale_state_read(st).found_inf == 1 and np.isposinf(np32(db)[17]) and np32(db)[0] == 4096.0
    big = 262144 + 8                     # one row block x this many columns: 8 floats too many
    assert mp.mp_colsum_workspace_bytes(64, big) > mp.mp_colsum_static_max_bytes()
    out = torch.full((big,), 5.0, dtype=torch.float16, device="cuda")
    with pytest.raises(mp.MPError) as e:
        mp.mp_colsum_static(64, big, torch.zeros(64, big, dtype=torch.float16, device="cuda"), big, out, None)
    assert e.value.code == ML.MP_E_WORKSPACE
    torch.cuda.synchronize()
    assert torch.all(out == 5.0)          # nothing was enqueued
    with pytest.raises(mp.MPError):
        mp.mp_colsum_static(0, 8, out, 8, out, None)
