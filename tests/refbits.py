"""Independent integer-only float32 -> binary16 round-to-nearest-even, used to pin
the oracle's storage rounding (which goes through NumPy's float16 cast).  Works on
uint32 bit patterns; no floating-point operation is involved."""
import numpy as np


def f32_to_f16_bits(x):
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    sign = ((u >> 16) & 0x8000).astype(np.uint64)
    exp = ((u >> 23) & 0xFF).astype(np.int64)
    man = (u & 0x7FFFFF).astype(np.uint64)
    out = np.zeros(u.shape, dtype=np.uint64)

    is_nan = (exp == 255) & (man != 0)
    is_inf = (exp == 255) & (man == 0)
    e16 = exp - 127 + 15                       # biased half exponent if normal

    # normal range candidates: keep 10 mantissa bits, round on the 13 dropped
    norm = (e16 >= 1) & (exp != 255)
    base = (e16.clip(0, 31).astype(np.uint64) << 10) | (man >> 13)
    rem = man & 0x1FFF
    up = (rem > 0x1000) | ((rem == 0x1000) & ((base & 1) == 1))
    nv = base + up.astype(np.uint64)           # carry may bump exponent; 0x7C00 = inf
    nv = np.where(nv >= 0x7C00, 0x7C00, nv)
    out = np.where(norm, nv, out)

    # subnormal / underflow: value = (2^23 + man) * 2^(exp-150); half subnormal unit 2^-24
    sub = (e16 < 1) & (exp != 255)
    full = man | np.where(exp > 0, 1 << 23, 0).astype(np.uint64)
    e_eff = np.where(exp > 0, exp, 1)
    shift = (126 - e_eff).astype(np.int64)     # result = full >> shift, 14 <= shift
    shift_c = shift.clip(0, 40).astype(np.uint64)
    q = full >> shift_c
    r = full & ((np.uint64(1) << shift_c) - np.uint64(1))
    half = np.uint64(1) << (shift_c - np.uint64(1))
    upc = (r > half) | ((r == half) & ((q & 1) == 1))
    sv = q + upc.astype(np.uint64)
    sv = np.where(shift > 40, 0, sv)
    out = np.where(sub, sv, out)

    out = np.where(is_inf, 0x7C00, out)
    out = np.where(is_nan, 0x7E00, out)
    return (out | sign).astype(np.uint16)
