"""Pins for the oracle's storage rounding and contraction arithmetic (CPU only)."""
import numpy as np
import pytest

from oracle import MIXED, FP32, FP64
from oracle import layers as L
from oracle.numerics import half_bits, from_half_bits
from refbits import f32_to_f16_bits


def test_store_is_rne_binary16_against_integer_routine():
    rng = np.random.default_rng(1)
    xs = [rng.standard_normal(200000).astype(np.float32) * np.float32(s)
          for s in (1e-9, 1e-7, 3e-5, 1e-3, 1.0, 300.0, 6e4, 1e6)]
    x = np.concatenate(xs)
    got = half_bits(MIXED.store(x))
    assert np.array_equal(got, f32_to_f16_bits(x))


def test_store_round_trips_every_half_pattern():
    bits = np.arange(65536, dtype=np.uint16)
    vals = from_half_bits(bits)
    back = half_bits(MIXED.store(vals))
    nan = np.isnan(vals)
    assert np.array_equal(back[~nan], bits[~nan])
    assert np.all(np.isnan(MIXED.store(vals[nan])))


def test_store_ties_and_range_edges():
    s = lambda v: float(MIXED.store(np.float32(v)))
    assert s(65520.0) == np.inf                    # tie between 65504 and 2^16 goes to even = overflow
    assert s(np.nextafter(np.float32(65520.0), np.float32(0))) == 65504.0
    assert s(-65520.0) == -np.inf
    assert s(2.0 ** -25) == 0.0                    # tie between 0 and the smallest subnormal -> even (0)
    assert s(np.nextafter(np.float32(2.0 ** -25), np.float32(1))) == 2.0 ** -24
    assert s(2.0 ** -24 * 1.5) == 2.0 ** -23       # tie 1.5 ulp -> even (2)
    assert s(1.0 + 2.0 ** -11) == 1.0              # tie to even mantissa
    assert s(1.0 + 3 * 2.0 ** -11) == 1.0 + 2.0 ** -9
    assert np.isnan(s(np.nan)) and s(np.inf) == np.inf


def test_fp32_fp64_policies_do_not_round():
    x = np.array([1.0 + 2.0 ** -20, 1e-30, 1e30])
    assert np.array_equal(FP64.store(x), x)
    assert FP32.store(x).dtype == np.float32 and FP32.store(x)[0] == np.float32(1.0 + 2.0 ** -20)


def _loops_linear(x, w, b):
    M, K = x.shape
    N = w.shape[0]
    y = np.zeros((M, N))
    for i in range(M):
        for j in range(N):
            acc = 0.0
            for k in range(K):
                acc += float(x[i, k]) * float(w[j, k])
            y[i, j] = acc + float(b[j])
    return y


def test_linear_brute_force_and_orientation():
    rng = np.random.default_rng(2)
    x = MIXED.store(rng.standard_normal((5, 7)))
    w = MIXED.store(rng.standard_normal((3, 7)))
    b = MIXED.store(rng.standard_normal(3))
    ref = _loops_linear(x, w, b)
    assert np.allclose(L.linear_fwd(FP64, FP64.island(x), FP64.island(w), FP64.island(b)), ref, rtol=0, atol=1e-13)
    # mixed result is the fp64 result rounded once (tiny sizes: fp32 accumulation error is far below 1/2 ulp16)
    got = L.linear_fwd(MIXED, x, w, b)
    assert np.array_equal(half_bits(got), f32_to_f16_bits(ref.astype(np.float32)))
    # backward orientation by brute force: dX = dY W, dW = dY^T X, db = column sums
    dy = MIXED.store(rng.standard_normal((5, 3)))
    dx, dw, db = L.linear_bwd(FP64, FP64.island(dy), FP64.island(x), FP64.island(w))
    dx_ref = np.array([[sum(dy[i, j] * w[j, k] for j in range(3)) for k in range(7)] for i in range(5)], dtype=np.float64)
    dw_ref = np.array([[sum(dy[i, j] * x[i, k] for i in range(5)) for k in range(7)] for j in range(3)], dtype=np.float64)
    assert np.allclose(dx, dx_ref, atol=1e-13) and np.allclose(dw, dw_ref, atol=1e-13)
    assert np.allclose(db, dy.sum(0), atol=1e-13)


def test_linear_identity_and_onehot_are_exact_copies():
    rng = np.random.default_rng(3)
    x = MIXED.store(rng.standard_normal((9, 16)))
    eye = np.eye(16, dtype=np.float32)
    assert np.array_equal(L.linear_fwd(MIXED, x, eye), x)
    perm = eye[rng.permutation(16)]
    assert np.array_equal(L.linear_fwd(MIXED, x, perm), x @ perm.T)
    y = L.linear_fwd(MIXED, x, eye, relu=True)
    assert np.array_equal(y, np.maximum(x, 0))


def test_fp16_products_are_exact_in_fp32_and_accumulation_is_fp32():
    rng = np.random.default_rng(4)
    a = MIXED.store(rng.standard_normal(4096) * 3)
    b = MIXED.store(rng.standard_normal(4096) * 3)
    assert np.array_equal((a * b).astype(np.float64), a.astype(np.float64) * b.astype(np.float64))
    # a long contraction: fp32-accumulated value agrees with fp64 to ~sqrt(K) 2^-24 relative to the
    # magnitude of the terms, i.e. it is NOT an fp16 accumulation (which would be off by ~1e-2).
    x = MIXED.store(rng.standard_normal((4, 8192)))
    w = MIXED.store(rng.standard_normal((6, 8192)))
    acc32 = (x @ w.T).astype(np.float64)
    acc64 = x.astype(np.float64) @ w.astype(np.float64).T
    assert np.max(np.abs(acc32 - acc64)) < 8192 ** 0.5 * 2.0 ** -22 * 4
    y = L.linear_fwd(MIXED, x, w)
    assert np.mean(half_bits(y) != f32_to_f16_bits(acc64.astype(np.float32))) <= 1 / 24


def test_overflow_becomes_inf_not_saturation():
    x = MIXED.store(np.full((1, 64), 200.0))
    w = MIXED.store(np.full((1, 64), 200.0))
    assert L.linear_fwd(MIXED, x, w)[0, 0] == np.inf       # 64 * 4e4 > 65504


def test_library_matmul_step_against_the_plain_ascending_k_contraction():
    """The oracle's contractions are NumPy matmuls (a BLAS routine that blocks and orders the fp32 sum as it likes).
    Section 3.1 only fixes "half-precision operands, single-precision sums", so any fp32 order is legitimate; this pins
    the library step against the literal statement (oracle/contract_plain.c: one fp32 accumulator per element, products
    in ascending k, no blocking) at the contraction lengths of the workloads: before the rounding to storage the two
    agree to fp32 reordering error (~sqrt(K) 2^-24 of the summed magnitudes), after it they are the same fp16 value
    except where that difference straddles a rounding boundary (then one ulp apart), and on operands whose partial sums
    are all exact in fp32 (small integers) they are bit-identical."""
    from oracle.contract_plain import contract_nt
    rng = np.random.default_rng(11)
    for (M, N, K) in ((64, 96, 256), (33, 130, 1024), (16, 64, 4096), (8, 40, 8192)):
        x, w = MIXED.store(rng.standard_normal((M, K))), MIXED.store(rng.standard_normal((N, K)) * 0.05)
        lib, plain = x @ w.T, contract_nt(x, w)
        scale = np.sqrt((x.astype(np.float64) ** 2) @ (w.astype(np.float64) ** 2).T)      # magnitude of the summed terms
        assert np.max(np.abs(lib - plain) / scale) < 8 * np.sqrt(K) * 2.0 ** -24
        truth = x.astype(np.float64) @ w.astype(np.float64).T
        assert np.max(np.abs(plain - truth) / scale) < 8 * np.sqrt(K) * 2.0 ** -24         # and both sit that close to the exact sum
        a, b = MIXED.store(lib), MIXED.store(plain)
        differ = a != b
        assert differ.mean() < 0.05
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(b), 2.0 ** -14))) - 10)
        assert np.all(np.abs(a - b)[differ] <= ulp[differ] * 1.001)
        # the layer function is that library step plus bias, ReLU and one rounding
        bias = MIXED.store(rng.standard_normal(N))
        y = L.linear_fwd(MIXED, x, w, bias, relu=True)
        y_plain = MIXED.store(np.maximum(plain + bias, np.float32(0)))
        assert (y != y_plain).mean() < 0.05 and np.linalg.norm(y - y_plain) <= 1e-4 * np.linalg.norm(y_plain)
    xi = rng.integers(-8, 9, (40, 512)).astype(np.float32)
    wi = rng.integers(-8, 9, (24, 512)).astype(np.float32)
    assert np.array_equal(xi @ wi.T, contract_nt(xi, wi))                                  # every partial sum exact: order cannot matter
    # orientation: the second operand is [N, K] (rows contract with rows)
    e = np.zeros((3, 5), np.float32); e[1, 2] = 1
    f = np.arange(20, dtype=np.float32).reshape(4, 5)
    assert np.array_equal(contract_nt(e, f), e @ f.T)
