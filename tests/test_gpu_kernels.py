"""Per-kernel parity of the HIP library (through its C ABI) against the CPU oracle, element by element,
on seeded inputs whose sizes span several tiles and ragged tails.  Tolerances (north-star): contraction and
gradient outputs rel. Frobenius <= 1e-3, fp32 masters <= 1e-5, flags and scale sequence exact."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_1805_10387_amd as mp
from paper_1805_10387_amd import _lib as ML
import mp_inputs as I
from oracle import MIXED
from oracle import layers as L
from oracle import optimizer as O
from oracle.numerics import half_bits
from gpu_util import *

RNG = lambda s: np.random.default_rng(1000 + s)
S16 = MIXED.store


def make_state(mode=ML.MP_SCALE_BACKOFF, scale=2.0 ** 15, interval=10, smin=1.0, smax=2.0 ** 24):
    st = mp.scale_state_alloc()
    mp.mp_scale_state_init(st, mode, scale, interval, smin, smax)
    return st


# ------------------------------------------------------------------ contractions
GEMM_SHAPES = [  # (M, N, K)
    (64, 1024, 256), (64, 256, 1024),          # config-1 layers
    (300, 200, 136), (257, 129, 72), (33, 520, 64), (512, 384, 1000), (8, 8, 8), (1, 40, 2048),
    (640, 512, 512),
]


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
@pytest.mark.parametrize("epi", ["none", "bias", "bias_relu"])
def test_gemm_fwd(M, N, K, epi):
    r = RNG(M + N + K)
    x, w, b = S16(r.standard_normal((M, K))), S16(r.standard_normal((N, K)) * 0.1), S16(r.standard_normal(N))
    ref = L.linear_fwd(MIXED, x, w, None if epi == "none" else b, relu=(epi == "bias_relu"))
    y = empty16(M, N)
    d = mp.gemm_desc(M, N, K, epilogue={"none": 0, "bias": 1, "bias_relu": 2}[epi])
    mp.mp_gemm_fwd(d, h16(x), h16(w), None if epi == "none" else h16(b), None, y)
    assert_close16(y, ref, 1e-3, max_ulp=1, what=f"fwd {M}x{N}x{K} {epi}")


@pytest.mark.parametrize("M,N,K", [(512, 384, 256), (300, 576, 136), (256, 192, 64), (1024, 3072, 128)])
def test_gemm_fwd_tile_256x192(M, N, K):
    """The 256 x 192 tile (contraction-contiguous operands only), forced: interior and ragged variants."""
    r = RNG(M + N + K + 5)
    x, w, b = S16(r.standard_normal((M, K))), S16(r.standard_normal((N, K)) * 0.1), S16(r.standard_normal(N))
    y = empty16(M, N)
    mp.mp_gemm_tuning_override(8, 1)
    try:
        mp.mp_gemm_fwd(mp.gemm_desc(M, N, K, epilogue=2), h16(x), h16(w), h16(b), None, y)
    finally:
        mp.mp_gemm_tuning_override(-1, 0)
    assert_close16(y, L.linear_fwd(MIXED, x, w, b, relu=True), 1e-3, max_ulp=1, what=f"fwd 256x192 tile {M}x{N}x{K}")


@pytest.mark.parametrize("tile,M,N,K", [(6, 1536, 1536, 1536), (6, 1536, 1536, 320), (6, 1536, 1536, 128),
                                        (3, 2560, 3456, 512), (0, 4352, 4096, 256)])
def test_gemm_workgroups_that_take_several_tiles(tile, M, N, K):
    """More tiles than resident workgroups: a workgroup goes on to a second tile, and with an even number (>= 4) of
    k-tiles the first k-tiles (and bias values) of that tile are fetched during the current one.  All three products,
    with the epilogues that read a second operand."""
    r = RNG(M + N + K + tile)
    x, w, b = S16(r.standard_normal((M, K))), S16(r.standard_normal((N, K)) * 0.1), S16(r.standard_normal(N))
    dy, src = S16(r.standard_normal((M, N))), S16(np.maximum(r.standard_normal((M, K)), 0))
    d = mp.gemm_desc(M, N, K, epilogue=2)
    y, dx, dw = empty16(M, N), empty16(M, K), empty16(N, K)
    st = make_state()
    ws = ws_bytes(mp.mp_gemm_bwd_dw_workspace_bytes(d, False))
    mp.mp_gemm_tuning_override(tile, 1)
    try:
        mp.mp_gemm_fwd(d, h16(x), h16(w), h16(b), None, y)
        mp.mp_gemm_bwd_dx(mp.gemm_desc(M, N, K), h16(dy), h16(w), dx, relu_src=h16(src), ld_aux=K)
        mp.mp_gemm_bwd_dw(mp.gemm_desc(M, N, K), h16(dy), h16(x), dw, None, st, ws)
    finally:
        mp.mp_gemm_tuning_override(-1, 0)
    assert_close16(y, L.linear_fwd(MIXED, x, w, b, relu=True), 1e-3, max_ulp=1, what="fwd")
    assert_close16(dx, L.relu_mask(MIXED, MIXED.store(dy @ w), src), 1e-3, max_ulp=1, what="dx")
    assert_close16(dw, MIXED.store(dy.T @ x), 1e-3, max_ulp=1, what="dw")
    assert mp.scale_state_read(st).found_inf == 0


@pytest.mark.parametrize("tile,M,N,K", [(0, 4352, 4096, 256), (0, 512, 512, 32), (0, 256, 768, 1056), (1, 2304, 1152, 96),
                                        (2, 1152, 2304, 160), (3, 2560, 3456, 512), (3, 128, 128, 32), (8, 512, 384, 224)])
def test_gemm_direct_to_lds_kernels_all_layouts(tile, M, N, K):
    """The kernels whose operand tiles go from global memory straight into LDS (ring of 32-deep k-tiles; transposing LDS
    reads for output-contiguous operands), forced for every product they are built for: forward (both operands
    contraction-contiguous), dX (second operand output-contiguous) and dW (both output-contiguous), every tile shape,
    one and several tiles per workgroup (the ring then runs on from tile to tile), k-tile counts below, at and above the
    ring depth, with the epilogues that read a second operand and the overflow flag."""
    r = RNG(M + N + K + tile + 3)
    x, w, b = S16(r.standard_normal((M, K))), S16(r.standard_normal((N, K)) * 0.1), S16(r.standard_normal(N))
    dy, src, other = S16(r.standard_normal((M, N))), S16(np.maximum(r.standard_normal((M, K)), 0)), S16(r.standard_normal((M, K)))
    d = mp.gemm_desc(M, N, K, epilogue=2)
    y, dx, dx2, dw = empty16(M, N), empty16(M, K), empty16(M, K), empty16(N, K)
    st = make_state()
    ws = ws_bytes(mp.mp_gemm_bwd_dw_workspace_bytes(d, False))
    mp.mp_gemm_tuning_override(tile, 1)
    mp.mp_gemm_tuning_dtl(2)
    try:
        mp.mp_gemm_fwd(d, h16(x), h16(w), h16(b), None, y)
        mp.mp_gemm_bwd_dx(mp.gemm_desc(M, N, K), h16(dy), h16(w), dx, relu_src=h16(src), ld_aux=K)
        mp.mp_gemm_bwd_dx(mp.gemm_desc(M, N, K), h16(dy), h16(w), dx2, add=h16(other), ld_aux=K)
        mp.mp_gemm_bwd_dw(mp.gemm_desc(M, N, K), h16(dy), h16(x), dw, None, st, ws)
    finally:
        mp.mp_gemm_tuning_override(-1, 0)
        mp.mp_gemm_tuning_dtl(1)
    assert_close16(y, L.linear_fwd(MIXED, x, w, b, relu=True), 1e-3, max_ulp=1, what="fwd")
    base = MIXED.store(dy @ w)
    assert_close16(dx, L.relu_mask(MIXED, base, src), 1e-3, max_ulp=1, what="dx relu")
    assert_close16(dx2, L.add_store(MIXED, base, other), 1e-3, what="dx add")
    assert_close16(dw, MIXED.store(dy.T @ x), 1e-3, max_ulp=1, what="dw")
    assert mp.scale_state_read(st).found_inf == 0
    # the same weight gradient with the kernels switched off: the register-staged path stays covered
    dw0 = empty16(N, K)
    mp.mp_gemm_tuning_override(tile if tile != 8 else 0, 1)
    mp.mp_gemm_tuning_dtl(0)
    try:
        mp.mp_gemm_bwd_dw(mp.gemm_desc(M, N, K), h16(dy), h16(x), dw0, None, st, ws)
    finally:
        mp.mp_gemm_tuning_override(-1, 0)
        mp.mp_gemm_tuning_dtl(1)
    assert_close16(dw0, MIXED.store(dy.T @ x), 1e-3, max_ulp=1, what="dw, register-staged")
    with pytest.raises(mp.MPError):
        mp.mp_gemm_tuning_dtl(3)


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_bwd_dx_and_dw(M, N, K):
    r = RNG(M * 3 + N + K)
    x, w = S16(r.standard_normal((M, K))), S16(r.standard_normal((N, K)) * 0.1)
    dy = S16(r.standard_normal((M, N)))
    dx_ref, dw_ref, db_ref = L.linear_bwd(MIXED, dy, x, w)
    d = mp.gemm_desc(M, N, K)
    dx = empty16(M, K)
    mp.mp_gemm_bwd_dx(d, h16(dy), h16(w), dx)
    assert_close16(dx, dx_ref, 1e-3, max_ulp=1, what="dx")
    dw, db = empty16(N, K), empty16(N)
    st = make_state()
    ws = ws_bytes(mp.mp_gemm_bwd_dw_workspace_bytes(d, True))
    mp.mp_gemm_bwd_dw(d, h16(dy), h16(x), dw, db, st, ws)
    assert_close16(dw, dw_ref, 1e-3, max_ulp=1, what="dw")
    assert_close16(db, db_ref, 1e-3, max_ulp=1, what="db")
    assert mp.scale_state_read(st).found_inf == 0


@pytest.mark.parametrize("M,N,K", [(64, 128, 64), (300, 264, 136), (70, 90, 50)])   # matrix-core interior, ragged, scalar path
def test_gemm_relu_epilogue_keeps_nonfinite_values(M, N, K):
    """max(x, 0) on a non-finite pre-activation: +inf stays +inf, -inf becomes 0 and NaN stays NaN, as in the
    oracle's definition.  A NaN that the epilogue dropped would hide a forward overflow from the gradient
    inspection (Section 3.1 item 1)."""
    r = RNG(M + N + K + 99)
    x, w, b = r.standard_normal((M, K)), r.standard_normal((N, K)) * 0.1, r.standard_normal(N)
    w[np.abs(w) < 1e-3] = 0.01                # (inf x 0 would make NaN on both sides, but keep the three cases apart)
    x[3, 5] = np.inf                          # row 3: +-inf by the sign of w[:, 5]
    x[7, 2] = np.nan                          # row 7: NaN everywhere
    x[9, 1], w[4, 1] = -np.inf, 0.0           # row 9: -+inf, and NaN where the weight is zero
    x, w, b = S16(x), S16(w), S16(b)
    with np.errstate(invalid="ignore"):
        ref = L.linear_fwd(MIXED, x, w, b, relu=True)
        ref_lin = L.linear_fwd(MIXED, x, w, b)
    assert np.isnan(ref[7]).all() and np.isnan(ref[9, 4]) and np.isposinf(ref[3]).any() and (ref[3] == 0).any()
    y = empty16(M, N)
    mp.mp_gemm_fwd(mp.gemm_desc(M, N, K, epilogue=2), h16(x), h16(w), h16(b), None, y)
    got = np32(y)
    assert np.array_equal(np.isnan(got), np.isnan(ref)) and np.array_equal(np.isposinf(got), np.isposinf(ref))
    assert not np.isneginf(got).any()
    assert_close16(y, ref, 1e-3, max_ulp=1, what="relu with non-finite inputs")
    mp.mp_gemm_fwd(mp.gemm_desc(M, N, K, epilogue=1), h16(x), h16(w), h16(b), None, y)
    got = np32(y)
    assert np.array_equal(np.isnan(got), np.isnan(ref_lin)) and np.array_equal(np.isneginf(got), np.isneginf(ref_lin))


def test_gemm_dx_relu_mask_and_residual_add():
    M, N, K = 200, 136, 264
    r = RNG(7)
    w, dy = S16(r.standard_normal((N, K)) * 0.1), S16(r.standard_normal((M, N)))
    src = S16(np.maximum(r.standard_normal((M, K)), 0))
    other = S16(r.standard_normal((M, K)))
    base = MIXED.store(dy @ w)
    d = mp.gemm_desc(M, N, K)
    out = empty16(M, K)
    mp.mp_gemm_bwd_dx(d, h16(dy), h16(w), out, relu_src=h16(src), ld_aux=K)
    assert_close16(out, L.relu_mask(MIXED, base, src), 1e-3, max_ulp=1, what="dx relu")
    assert np.all(np32(out)[src <= 0] == 0)
    mp.mp_gemm_bwd_dx(d, h16(dy), h16(w), out, add=h16(other), ld_aux=K)
    # one ulp of the intermediate rounding can exceed one ulp of the (possibly cancelling) sum: norm bound only
    assert_close16(out, L.add_store(MIXED, base, other), 1e-3, what="dx add")


def test_gemm_leading_dimensions_and_unaligned_fallback():
    r = RNG(8)
    M, N, K = 70, 90, 50                      # K, N not multiples of 8: slow path
    x, w = S16(r.standard_normal((M, K))), S16(r.standard_normal((N, K)))
    y = empty16(M, N)
    mp.mp_gemm_fwd(mp.gemm_desc(M, N, K), h16(x), h16(w), None, None, y)
    assert_close16(y, L.linear_fwd(MIXED, x, w), 1e-3, max_ulp=1, what="unaligned")
    # ld > cols, aligned: views into wider buffers
    M, N, K = 96, 72, 40
    xb, wb = S16(r.standard_normal((M, 64))), S16(r.standard_normal((N, 48)))
    yb = torch.full((M, 80), 7.0, dtype=torch.float16, device="cuda")
    mp.mp_gemm_fwd(mp.gemm_desc(M, N, K, ldx=64, ldw=48, ldy=80), h16(xb), h16(wb), None, None, yb)
    assert_close16(yb[:, :N], L.linear_fwd(MIXED, xb[:, :K], wb[:, :K]), 1e-3, max_ulp=1, what="ld")
    assert torch.all(yb[:, N:] == 7.0)        # nothing written outside the N columns


def test_gemm_fp32_addend_and_fp32_output():
    r = RNG(9)
    M, N, K1, K2 = 48, 264, 136, 72
    x1, x2 = S16(r.standard_normal((M, K1))), S16(r.standard_normal((M, K2)))
    w = S16(r.standard_normal((N, K1 + K2)) * 0.2)
    b = S16(r.standard_normal(N))
    ref = L.linear_fwd(MIXED, np.concatenate([x1, x2], 1), w, b)
    part = empty32(M, N)
    wd = h16(w)
    mp.mp_gemm_fwd(mp.gemm_desc(M, N, K1, ldw=K1 + K2), h16(x1), wd, None, None, None, part)
    y = empty16(M, N)
    mp.mp_gemm_fwd(mp.gemm_desc(M, N, K2, ldw=K1 + K2, epilogue=1), h16(x2), wd[:, K1:], h16(b), part, y)
    assert_close16(y, ref, 1e-3, max_ulp=1, what="split contraction")


def test_gemm_attention_batched_strided():
    """Q K^T, P V and their gradients on a fused qkv buffer, batch = (sequence, head), no copies."""
    B, S, h, dk = 3, 40, 4, 64
    d_model, T = h * dk, B * S
    r = RNG(10)
    qkv = S16(r.standard_normal((T, 3 * d_model)))
    ctx_ref, cache = L.attention_fwd(MIXED, qkv, B, S, h)
    q, k, v, p, alpha = cache
    qkv_d = h16(qkv)
    s_d = empty16(B, h, S, S)
    ds = mp.gemm_desc(S, S, dk, ldx=3 * d_model, ldw=3 * d_model, ldy=S, alpha=float(alpha), batch_outer=B, batch_inner=h,
                      sx=(S * 3 * d_model, dk), sw=(S * 3 * d_model, dk), sy=(h * S * S, S * S))
    mp.mp_gemm_fwd(ds, qkv_d, qkv_d[:, d_model:], None, None, s_d)
    s_ref = MIXED.store(alpha * (q @ k.transpose(0, 1, 3, 2)))
    assert_close16(s_d, s_ref, 1e-3, max_ulp=1, what="scores")
    p_d = empty16(B, h, S, S)
    mp.mp_softmax_fwd(B * h * S, S, s_d, p_d, S)
    assert_close16(p_d, p, 1e-3, max_ulp=2, what="softmax")
    ctx_d = empty16(T, d_model)
    dc = mp.gemm_desc(S, dk, S, ldx=S, ldw=3 * d_model, ldy=d_model, trans_w=1, batch_outer=B, batch_inner=h,
                      sx=(h * S * S, S * S), sw=(S * 3 * d_model, dk), sy=(S * d_model, dk))
    mp.mp_gemm_fwd(dc, p_d, qkv_d[:, 2 * d_model:], None, None, ctx_d)
    assert_close16(ctx_d, ctx_ref, 1e-3, what="ctx")
    # backward (from the oracle's p so that the comparison isolates these kernels)
    dctx = S16(r.standard_normal((T, d_model)))
    dqkv_ref = L.attention_bwd(MIXED, dctx, cache)
    p_o, dctx_d = h16(p), h16(dctx)
    dp_d, dqkv_d = empty16(B, h, S, S), empty16(T, 3 * d_model)
    ws = ws_bytes(1 << 20)
    mp.mp_gemm_bwd_dx(dc, dctx_d, qkv_d[:, 2 * d_model:], dp_d)                     # dP = dctx V^T
    mp.mp_gemm_bwd_dw(dc, dctx_d, p_o, dqkv_d[:, 2 * d_model:], None, None, ws)      # dV = P^T dctx
    ds_d = empty16(B, h, S, S)
    mp.mp_softmax_bwd(B * h * S, S, p_o, dp_d, ds_d, S)
    mp.mp_gemm_bwd_dx(ds, ds_d, qkv_d[:, d_model:], dqkv_d)                          # dQ = alpha dS K
    mp.mp_gemm_bwd_dw(ds, ds_d, qkv_d, dqkv_d[:, d_model:], None, None, ws)          # dK = alpha dS^T Q
    assert_close16(dqkv_d, dqkv_ref, 1e-3, what="dqkv")


@pytest.mark.parametrize("B,S,h", [(3, 128, 2), (2, 40, 3), (5, 64, 1), (1, 8, 4), (2, 104, 2)])
def test_fused_attention_fwd_bwd(B, S, h):
    dk = 64
    d_model, T = h * dk, B * S
    r = RNG(B * 1000 + S + h)
    qkv = S16(r.standard_normal((T, 3 * d_model)))
    ctx_ref, cache = L.attention_fwd(MIXED, qkv, B, S, h)
    q, k, v, p_ref, alpha = cache
    qkv_d = h16(qkv)
    p_d = torch.zeros(B, h, S, S, dtype=torch.float16, device="cuda")
    ctx_d = torch.full((T, d_model + 8), 3.0, dtype=torch.float16, device="cuda")
    mp.mp_attention_fwd(B, h, S, dk, qkv_d, 3 * d_model, float(alpha), p_d, ctx_d, d_model + 8)
    assert_close16(p_d, p_ref, 1e-3, max_ulp=2, what="fused p")
    assert_close16(ctx_d[:, :d_model], ctx_ref, 1e-3, what="fused ctx")
    assert torch.all(ctx_d[:, d_model:] == 3.0)
    # backward from the GPU's own p (the stored tensor both sides would use)
    dctx = S16(r.standard_normal((T, d_model)))
    p_gpu = np32(p_d)
    dqkv_ref = L.attention_bwd(MIXED, dctx, (q, k, v, p_gpu, alpha))
    dqkv_d = torch.zeros(T, 3 * d_model, dtype=torch.float16, device="cuda")
    mp.mp_attention_bwd(B, h, S, dk, qkv_d, 3 * d_model, float(alpha), p_d, h16(dctx), d_model, dqkv_d, 3 * d_model)
    for name, lo in (("dq", 0), ("dk", d_model), ("dv", 2 * d_model)):
        assert_close16(dqkv_d[:, lo:lo + d_model], dqkv_ref[:, lo:lo + d_model], 1e-3, what=f"fused {name}")


def test_fused_attention_rejects_unsupported_shapes():
    x = empty16(64, 3 * 96)
    with pytest.raises(mp.MPError) as e:
        mp.mp_attention_fwd(1, 2, 64, 48, x, 3 * 96, 0.1, empty16(1, 2, 64, 64), empty16(64, 96), 96)
    assert e.value.code == ML.MP_E_UNSUPPORTED
    x = empty16(36, 3 * 64)
    with pytest.raises(mp.MPError):
        mp.mp_attention_fwd(1, 1, 36, 64, x, 3 * 64, 0.1, empty16(1, 1, 36, 36), empty16(36, 64), 64)


def test_gemm_overflow_gives_inf_and_dw_sets_flag():
    M, N, K = 64, 64, 64
    x = np.full((M, K), 200.0, np.float32)
    w = np.full((N, K), 200.0, np.float32)
    y = empty16(M, N)
    mp.mp_gemm_fwd(mp.gemm_desc(M, N, K), h16(x), h16(w), None, None, y)
    assert np.all(np.isposinf(np32(y)))                   # 64 * 4e4 overflows fp16: inf, never 65504
    st = make_state()
    d = mp.gemm_desc(M, N, K)
    dw = empty16(N, K)
    ws = ws_bytes(mp.mp_gemm_bwd_dw_workspace_bytes(d, False))
    mp.mp_gemm_bwd_dw(d, h16(x), h16(w), dw, None, st, ws)
    assert mp.scale_state_read(st).found_inf == 1


def test_gemm_split_k_weight_gradient():
    M, N, K = 4096, 128, 256                  # small output, long token contraction: split over K
    r = RNG(11)
    x, dy = S16(r.standard_normal((M, K))), S16(r.standard_normal((M, N)) * 0.05)
    d = mp.gemm_desc(M, N, K)
    dw, db = empty16(N, K), empty16(N)
    ws = ws_bytes(mp.mp_gemm_bwd_dw_workspace_bytes(d, True))
    mp.mp_gemm_bwd_dw(d, h16(dy), h16(x), dw, db, None, ws)
    _, dw_ref, db_ref = L.linear_bwd(MIXED, dy, x, np.zeros((N, K), np.float32))
    assert_close16(dw, dw_ref, 1e-3, max_ulp=1, what="split-K dw")
    assert_close16(db, db_ref, 1e-3, max_ulp=1, what="db")


@pytest.mark.parametrize("shapes", [
    [(192, 256, 128), (192, 128, 384), (192, 384, 256)],      # multiples of 128 only: 128 x 128 tiles
    [(128, 256, 512), (128, 512, 256), (128, 256, 256)],      # multiples of 256: 256 x 256 tiles
    [(320, 1024, 256)] * 5,                                     # more tiles than workgroups resident at once
])
def test_gemm_grouped_weight_gradients(shapes):
    """Several dW = dY^T X in one launch: each equals the oracle and, bit for bit, the single-problem entry point."""
    r = RNG(len(shapes) * 7 + shapes[0][1])
    items, refs, singles, db_refs = [], [], [], []
    st = make_state()
    all256 = all(n % 256 == 0 and k % 256 == 0 for (_, n, k) in shapes)
    for j, (M, N, K) in enumerate(shapes):
        x, dy = S16(r.standard_normal((M, K))), S16(r.standard_normal((M, N)) * 0.1)
        d = mp.gemm_desc(M, N, K)
        dw, dw1 = empty16(N, K), empty16(N, K)
        # every item but the second also asks for its bias gradient from the same launch
        items.append((d, h16(dy), h16(x), dw) + ((empty16(N),) if j != 1 else ()))
        _, dw_ref, db_ref = L.linear_bwd(MIXED, dy, x, np.zeros((N, K), np.float32))
        refs.append(dw_ref)
        db_refs.append(db_ref)
        mp.mp_gemm_tuning_override(0 if all256 else 3, 1)         # the tile the grouped launch takes, no k-split
        mp.mp_gemm_bwd_dw(d, items[-1][1], items[-1][2], dw1, None, None, ws_bytes(mp.mp_gemm_bwd_dw_workspace_bytes(d, False)))
        mp.mp_gemm_tuning_override(-1, 0)
        singles.append(dw1)
    for mode in (1, 0):                                           # direct-to-LDS kernels (built-in choice), register-staged kernels
        mp.mp_gemm_tuning_dtl(mode)
        try:
            for it in items:
                for out in it[3:]:
                    out.fill_(float("nan"))
            mp.mp_gemm_bwd_dw_grouped(mp.gemm_group(items), st)
        finally:
            mp.mp_gemm_tuning_dtl(1)
        for k, (it, ref, one) in enumerate(zip(items, refs, singles)):
            assert_close16(it[3], ref, 1e-3, max_ulp=1, what=f"grouped dw {k} (mode {mode})")
            assert torch.equal(it[3], one), f"grouped dw {k} differs from the single-problem result (mode {mode})"
            if len(it) > 4:
                assert_close16(it[4], db_refs[k], 1e-3, max_ulp=1, what=f"grouped db {k} (mode {mode})")
    assert mp.scale_state_read(st).found_inf == 0


def test_gemm_grouped_transposed_weight_layout_with_bias_gradient():
    """A grouped item whose weight is stored [K, N] (trans_w): dW[K, N] = X^T dY, and db = column sums of dY, next to an
    ordinary item; both kernel families."""
    r = RNG(77)
    M, N, K = 192, 256, 384
    x, dy = S16(r.standard_normal((M, K))), S16(r.standard_normal((M, N)) * 0.1)
    _, dw_ref, db_ref = L.linear_bwd(MIXED, dy, x, np.zeros((N, K), np.float32))
    dt = mp.gemm_desc(M, N, K, ldw=N, trans_w=1)
    dn = mp.gemm_desc(M, N, K)
    for mode in (1, 0):
        dwt, dbt, dwn = empty16(K, N), empty16(N), empty16(N, K)
        for t in (dwt, dbt, dwn):
            t.fill_(float("nan"))
        mp.mp_gemm_tuning_dtl(mode)
        try:
            mp.mp_gemm_bwd_dw_grouped(mp.gemm_group([(dt, h16(dy), h16(x), dwt, dbt), (dn, h16(dy), h16(x), dwn)]), None)
        finally:
            mp.mp_gemm_tuning_dtl(1)
        assert_close16(dwt, dw_ref.T, 1e-3, max_ulp=1, what=f"grouped dw, [K, N] layout (mode {mode})")
        assert_close16(dwn, dw_ref, 1e-3, max_ulp=1, what=f"grouped dw (mode {mode})")
        assert_close16(dbt, db_ref, 1e-3, max_ulp=1, what=f"grouped db (mode {mode})")


def test_gemm_grouped_flags_overflow_and_rejects_ragged_shapes():
    M, N, K = 128, 128, 128
    big = torch.full((M, N), 300.0, dtype=torch.float16, device="cuda")
    x = torch.full((M, K), 300.0, dtype=torch.float16, device="cuda")
    ok_dy, ok_x = torch.ones(M, N, dtype=torch.float16, device="cuda"), torch.ones(M, K, dtype=torch.float16, device="cuda")
    st = make_state()
    d = mp.gemm_desc(M, N, K)
    dw0, dw1 = empty16(N, K), empty16(N, K)
    mp.mp_gemm_bwd_dw_grouped(mp.gemm_group([(d, ok_dy, ok_x, dw0), (d, big, x, dw1)]), st)
    assert mp.scale_state_read(st).found_inf == 1          # 128 * 300 * 300 overflows fp16
    assert torch.all(dw0 == 128.0) and torch.all(torch.isinf(dw1))
    # a bias gradient that overflows while the product stays finite: 128 rows of 600 sum to 76800 > 65504
    st2 = make_state()
    dy600 = torch.full((M, N), 600.0, dtype=torch.float16, device="cuda")
    zeros, db = torch.zeros(M, K, dtype=torch.float16, device="cuda"), empty16(N)
    mp.mp_gemm_bwd_dw_grouped(mp.gemm_group([(d, dy600, zeros, dw0, db)]), st2)
    assert mp.scale_state_read(st2).found_inf == 1 and torch.all(dw0 == 0.0) and torch.all(torch.isinf(db))
    bad = mp.gemm_desc(128, 136, 128)
    with pytest.raises(mp.MPError) as e:
        mp.mp_gemm_bwd_dw_grouped(mp.gemm_group([(bad, empty16(128, 136), ok_x, empty16(136, 128))]), st)
    assert e.value.code == ML.MP_E_UNSUPPORTED


def test_mfma_sustained_rate_probe_reads_sanely():
    """The ceiling probe: all-zero operands run near the top clock, N(0,1) operands clearly below it, both far above
    anything a memory-bound loop could show; the sink receives the (finite) accumulator sums."""
    sink = empty32(256 * 256)
    zeros = torch.zeros(16384, dtype=torch.float16, device="cuda")
    normal = torch.randn(16384, device="cuda", generator=torch.Generator(device="cuda").manual_seed(3)).half()
    r0 = mp.mp_mfma_sustained_rate(zeros, sink, 256, 20000)
    assert torch.all(sink == 0)
    r1 = mp.mp_mfma_sustained_rate(normal, sink, 256, 20000)
    assert torch.isfinite(sink).all()
    assert r0 > 0 and 0.3 * r0 < r1 < r0, (r0, r1)       # ratios only: absolute rates depend on the box's clocks


@pytest.mark.parametrize("M,N,K", [(32, 4096, 2048), (32, 1024, 512), (8, 2048, 4096), (48, 520, 1000)])
def test_gemm_few_rows_with_workspace(M, N, K):
    """Products with few output rows (the recurrent products of config 5) given a workspace: the contraction may be
    split over more workgroups; forward with and without bias and dX against the oracle, also with a workspace that
    is too small (runs unsplit) and with an epilogue that is never split (ReLU)."""
    r = RNG(M + N + K + 17)
    x, w, b = S16(r.standard_normal((M, K))), S16(r.standard_normal((N, K)) * 0.05), S16(r.standard_normal(N))
    dy = S16(r.standard_normal((M, N)))
    d0, d1, d2 = mp.gemm_desc(M, N, K), mp.gemm_desc(M, N, K, epilogue=1), mp.gemm_desc(M, N, K, epilogue=2)
    need = mp.mp_gemm_split_workspace_bytes(d0)
    if (M, N, K) == (32, 4096, 2048):
        assert need > 0                                       # this one must split, or config 5 stays latency-bound
    xd, wd, bd, dyd = h16(x), h16(w), h16(b), h16(dy)
    for ws in (ws_bytes(max(need, 256)), ws_bytes(256), None):
        y = empty16(M, N)
        mp.mp_gemm_fwd_ws(d0, xd, wd, None, None, y, ws=ws)
        assert_close16(y, L.linear_fwd(MIXED, x, w), 1e-3, max_ulp=1, what="few rows fwd")
        mp.mp_gemm_fwd_ws(d1, xd, wd, bd, None, y, ws=ws)
        assert_close16(y, L.linear_fwd(MIXED, x, w, b), 1e-3, max_ulp=1, what="few rows fwd + bias")
        mp.mp_gemm_fwd_ws(d2, xd, wd, bd, None, y, ws=ws)
        assert_close16(y, L.linear_fwd(MIXED, x, w, b, relu=True), 1e-3, max_ulp=1, what="few rows fwd + bias + relu")
        dx = empty16(M, K)
        mp.mp_gemm_bwd_dx_ws(d0, dyd, wd, dx, ws=ws)
        assert_close16(dx, L.linear_bwd(MIXED, dy, x, w)[0], 1e-3, max_ulp=1, what="few rows dx")


def test_empty_and_degenerate_inputs():
    """Zero rows: nothing is launched and the output is untouched.  Zero-length contraction: the sum is empty, the
    epilogue still applies (Y = bias).  An empty tensor list and zero-length tensors in the optimizer wrapper: the step
    counts as clean and the scale state advances like the oracle's."""
    y = torch.full((4, 8), 3.0, dtype=torch.float16, device="cuda")
    x, w = empty16(4, 8), empty16(8, 8)
    mp.mp_gemm_fwd(mp.gemm_desc(0, 8, 8), x, w, None, None, y)
    torch.cuda.synchronize()
    assert torch.all(y == 3.0)
    b = h16(S16(RNG(3).standard_normal(8)))
    mp.mp_gemm_fwd(mp.gemm_desc(4, 8, 0, ldx=8, ldw=8, epilogue=1), x, w, b, None, y)
    assert torch.equal(y, b.expand(4, 8))
    dx = torch.full((4, 8), 5.0, dtype=torch.float16, device="cuda")
    mp.mp_gemm_bwd_dx(mp.gemm_desc(4, 0, 8, ldy=8), empty16(4, 8), empty16(8, 8), dx)     # no output columns to contract over
    assert torch.all(dx == 0)
    st = make_state(interval=2)
    cfg = mp.opt_cfg("adam", 1e-3)
    mp.mp_unscale_check_update(None, 0, cfg, st)
    mp.mp_loss_scale_update(st)
    one = dict(g16=h16(np.ones(16, np.float32)), w32=f32(np.ones(16, np.float32)), w16=empty16(16), m=f32(np.zeros(16, np.float32)),
               v=f32(np.zeros(16, np.float32)))
    lst = mp.tensor_list([one, one])
    lst[0].n = 0                                             # a zero-length tensor in front of a real one
    mp.mp_unscale_check_update(lst, 2, cfg, st)
    mp.mp_loss_scale_update(st)
    s = mp.scale_state_read(st)
    ost = O.ScaleState(scale=2.0 ** 15, growth_interval=2)
    O.loss_scale_update(ost, 0)
    O.loss_scale_update(ost, 0)
    assert (s.scale, s.good_steps, s.opt_step, s.skipped_steps) == (ost.scale, ost.good_steps, ost.opt_step, 0) and s.scale == 2.0 ** 16
    assert torch.all(one["w32"] < 1.0) and torch.equal(one["w16"], one["w32"].half())


def test_gemm_rejects_bad_arguments():
    d = mp.gemm_desc(8, 8, 8)
    with pytest.raises(mp.MPError) as e:
        mp.mp_gemm_fwd(d, None, None, None, None, None)
    assert e.value.code == ML.MP_E_INVAL
    d2 = mp.gemm_desc(8, 8, 8, ldx=4)
    with pytest.raises(mp.MPError):
        mp.mp_gemm_fwd(d2, empty16(8, 8), empty16(8, 8), None, None, empty16(8, 8))
    with pytest.raises(mp.MPError) as e:
        mp.mp_gemm_bwd_dw(d, empty16(8, 8), empty16(8, 8), empty16(8, 8), None, None, None)
    assert e.value.code == ML.MP_E_WORKSPACE


# ------------------------------------------------------------------ losses
@pytest.mark.parametrize("rows,cols", [(64, 256), (37, 100), (1, 8), (513, 1000)])
def test_mse_scaled(rows, cols):
    r = RNG(rows + cols)
    y, t = S16(r.standard_normal((rows, cols))), S16(r.standard_normal((rows, cols)))
    S = 2.0 ** 10
    loss_ref, dy_ref = L.mse_scaled(MIXED, y, t, S)
    st = make_state(scale=S)
    loss, dy = empty32(1), empty16(rows, cols)
    mp.mp_mse_scaled(rows, cols, h16(y), h16(t), cols, st, loss, dy, ws_bytes(mp.mp_loss_workspace_bytes(rows, cols)))
    assert abs(float(loss) - float(loss_ref)) <= 1e-5 * abs(float(loss_ref))
    assert_close16(dy, dy_ref, 1e-3, max_ulp=1, what="mse dy")


@pytest.mark.parametrize("rows,vocab", [(16, 32768), (33, 3000), (7, 1001), (5, 40000),
                                        (600, 32768), (300, 24584)])  # the last two: several rows per persistent workgroup
def test_softmax_xent_scaled(rows, vocab):
    r = RNG(rows + vocab)
    z = S16(r.standard_normal((rows, vocab)) * 3)
    t = r.integers(0, vocab, rows).astype(np.int32)
    if rows > 4:
        t[1], t[2] = -1, vocab                # out-of-range targets contribute nothing
    S = 2.0 ** 15
    loss_ref, g_ref = L.softmax_xent_scaled(MIXED, z, t, S)
    st = make_state(scale=S)
    loss, g = empty32(1), empty16(rows, vocab)
    ws = ws_bytes(mp.mp_loss_workspace_bytes(rows, vocab))
    zd = h16(z)
    mp.mp_softmax_xent_scaled(rows, vocab, zd, vocab, i32(t), st, loss, g, ws)
    assert abs(float(loss) - float(loss_ref)) <= 2e-6 * abs(float(loss_ref)) + 1e-6
    assert_close16(g, g_ref, 1e-3, max_ulp=2, what="xent grad")
    mp.mp_softmax_xent_scaled(rows, vocab, zd, vocab, i32(t), st, loss, zd, ws)   # in place
    assert np.array_equal(bits(zd), bits(g))


@pytest.mark.parametrize("rows,vocab", [(600, 32768), (300, 24584), (16, 32768), (33, 3000), (7, 1001)])
def test_softmax_xent_scaled_with_bias_gradient(rows, vocab):
    """The loss call that also sums the stored gradient per column (the bias gradient of the projection): same loss and
    the same gradient bits as the plain call, db equal to the oracle's column sums of that gradient; the first two shapes
    take the fused pass (several rows per persistent workgroup), the others the plain call followed by mp_colsum."""
    r = RNG(3 * rows + vocab)
    z = S16(r.standard_normal((rows, vocab)) * 3)
    t = r.integers(0, vocab, rows).astype(np.int32)
    t[1], t[2] = -1, vocab
    S = 2.0 ** 15
    loss_ref, g_ref = L.softmax_xent_scaled(MIXED, z, t, S)
    db_ref = L.linear_bwd(MIXED, g_ref, np.zeros((rows, 8), np.float32), np.zeros((vocab, 8), np.float32))[2]
    st = make_state(scale=S)
    loss, loss2, g, g2, db = empty32(1), empty32(1), empty16(rows, vocab), empty16(rows, vocab), empty16(vocab)
    db.fill_(float("nan"))
    zd = h16(z)
    mp.mp_softmax_xent_scaled(rows, vocab, zd, vocab, i32(t), st, loss, g, ws_bytes(mp.mp_loss_workspace_bytes(rows, vocab)))
    ws = ws_bytes(mp.mp_softmax_xent_db_workspace_bytes(rows, vocab))
    mp.mp_softmax_xent_scaled_db(rows, vocab, zd, vocab, i32(t), st, loss2, g2, db, ws)
    assert float(loss2) == float(loss) and np.array_equal(bits(g2), bits(g))
    assert abs(float(loss2) - float(loss_ref)) <= 2e-6 * abs(float(loss_ref)) + 1e-6
    # column sums of the gradient the GPU stored (its own bits), and of the oracle's gradient
    own = L.linear_bwd(MIXED, np32(g2), np.zeros((rows, 8), np.float32), np.zeros((vocab, 8), np.float32))[2]
    assert_close16(db, own, 1e-3, max_ulp=1, what="xent db vs sums of the stored gradient")
    assert_close16(db, db_ref, 2e-3, max_ulp=4, what="xent db vs oracle")
    assert mp.scale_state_read(st).found_inf == 0
    mp.mp_softmax_xent_scaled_db(rows, vocab, zd, vocab, i32(t), st, loss2, zd, db, ws)   # in place
    assert np.array_equal(bits(zd), bits(g))
    with pytest.raises(mp.MPError) as e:
        mp.mp_softmax_xent_scaled_db(rows, vocab, zd, vocab, i32(t), st, loss2, zd, db, ws_bytes(1024))
    assert e.value.code == ML.MP_E_WORKSPACE


def test_softmax_xent_bias_gradient_flags_overflow():
    """Every row has the same target and a dominant logit elsewhere: the column of the dominant class sums
    rows x S / rows = S = 2^17 > 65504, so db overflows while every stored gradient value is small."""
    rows, vocab = 512, 32768
    z = torch.zeros(rows, vocab, dtype=torch.float16, device="cuda")
    z[:, 7] = 30.0
    st = make_state(scale=2.0 ** 17)
    loss, db = empty32(1), empty16(vocab)
    mp.mp_softmax_xent_scaled_db(rows, vocab, z, vocab, i32(np.full(rows, 3)), st, loss, z, db,
                                 ws_bytes(mp.mp_softmax_xent_db_workspace_bytes(rows, vocab)))
    assert mp.scale_state_read(st).found_inf == 1
    assert torch.isinf(db[7]) and torch.isfinite(z).all()


def test_xent_uniform_logits_closed_form():
    rows, vocab = 8, 32768
    st = make_state(scale=2.0 ** 15)
    loss, g = empty32(1), empty16(rows, vocab)
    z = torch.zeros(rows, vocab, dtype=torch.float16, device="cuda")
    mp.mp_softmax_xent_scaled(rows, vocab, z, vocab, i32(np.arange(rows)), st, loss, g,
                              ws_bytes(mp.mp_loss_workspace_bytes(rows, vocab)))
    assert abs(float(loss) - 10.39720770839918) < 1e-5          # ln 32768


# ------------------------------------------------------------------ LayerNorm / softmax / LSTM cell / colsum / cast
@pytest.mark.parametrize("rows,d", [(64, 512), (203, 1024), (5, 8), (130, 2048), (31, 200)])
def test_layernorm_fwd_bwd(rows, d):
    r = RNG(rows + d)
    x, a = S16(r.standard_normal((rows, d))), S16(r.standard_normal((rows, d)) * 0.5)
    gam, bet = S16(1 + 0.2 * r.standard_normal(d)), S16(0.1 * r.standard_normal(d))
    dy = S16(r.standard_normal((rows, d)))
    y_ref, cache = L.layernorm_fwd(MIXED, x, a, gam, bet)
    dz_ref, dg_ref, db_ref = L.layernorm_bwd(MIXED, dy, cache, gam)
    xd, ad, gd, bd = h16(x), h16(a), h16(gam), h16(bet)
    y, mean, rstd = empty16(rows, d), empty32(rows), empty32(rows)
    mp.mp_layernorm_fwd(rows, d, xd, ad, gd, bd, L.LN_EPS, y, mean, rstd)
    assert_close16(y, y_ref, 1e-3, max_ulp=1, what="ln y")
    assert np.allclose(np32(rstd), cache[1][:, 0], rtol=1e-5)
    dz, dg, db, dzs = empty16(rows, d), empty16(d), empty16(d), empty16(d)
    st = make_state()
    mp.mp_layernorm_bwd(rows, d, h16(dy), xd, ad, gd, mean, rstd, dz, dg, db, st,
                        ws_bytes(mp.mp_layernorm_bwd_workspace_bytes(rows, d)), dz_colsum=dzs)
    assert_close16(dz, dz_ref, 1e-3, what="ln dz")
    # the fused column sums are those of the dz the kernel stored
    assert_close16(dzs, MIXED.store(np32(dz).sum(0, dtype=np.float32)), 1e-3, max_ulp=1, what="ln dz colsum")
    dg2, db2 = empty16(d), empty16(d)
    mp.mp_layernorm_bwd(rows, d, h16(dy), xd, ad, gd, mean, rstd, dz, dg2, db2, None,
                        ws_bytes(mp.mp_layernorm_bwd_workspace_bytes(rows, d)))
    assert np.array_equal(bits(dg2), bits(dg)) and np.array_equal(bits(db2), bits(db))
    assert_close16(dg, dg_ref, 1e-3, max_ulp=1, what="ln dgamma")
    assert_close16(db, db_ref, 1e-3, max_ulp=1, what="ln dbeta")
    assert mp.scale_state_read(st).found_inf == 0


@pytest.mark.parametrize("rows,cols", [(64, 64), (1000, 128), (77, 40), (50, 256), (9, 512), (13, 301), (6, 1000)])
def test_softmax_fwd_bwd(rows, cols):
    r = RNG(rows + cols)
    s = S16(r.standard_normal((rows, cols)) * 2)
    p_ref = MIXED.store(L.softmax_rows(MIXED, s))
    p = empty16(rows, cols)
    mp.mp_softmax_fwd(rows, cols, h16(s), p, cols)
    assert_close16(p, p_ref, 1e-3, max_ulp=2, what="softmax")
    dp = S16(r.standard_normal((rows, cols)))
    inner = (dp * p_ref).sum(-1, keepdims=True, dtype=np.float32)
    ds_ref = MIXED.store(p_ref * (dp - inner))
    ds = empty16(rows, cols)
    mp.mp_softmax_bwd(rows, cols, h16(p_ref), h16(dp), ds, cols)
    assert_close16(ds, ds_ref, 1e-3, what="softmax bwd")


@pytest.mark.parametrize("B,H", [(32, 1024), (8, 128), (3, 50)])
def test_lstm_cell_fwd_bwd(B, H):
    """The cell kernels against the oracle's LSTM layer itself.  With W = [I_4H | 0] (input width 4H) and b = 0 the
    layer's gate sums are its inputs (an exact copy), the recurrent gradient is zero and dx_t = dgates_t, so a
    two-step sequence exposes one cell update with c_prev = 0 and one with c_prev != 0, and backward steps with and
    without an incoming cell-state gradient."""
    r = RNG(B + H)
    T = 2
    x_seq = S16(r.standard_normal((T, B, 4 * H)) * 2)
    w = np.concatenate([np.eye(4 * H, dtype=np.float32), np.zeros((4 * H, H), np.float32)], axis=1)
    h_ref, cache = L.lstm_layer_fwd(MIXED, x_seq, w, np.zeros(4 * H, np.float32))
    _, gates_all, c_all, _ = cache
    assert np.array_equal(gates_all, x_seq)
    gd = h16(x_seq)
    c = [torch.zeros(B, H, dtype=torch.float32, device="cuda"), empty32(B, H), empty32(B, H)]
    h1 = empty16(T, B, H)
    h2 = torch.zeros(T, B, 2 * H + 8, dtype=torch.float16, device="cuda")
    for t in range(T):
        mp.mp_lstm_cell_fwd(B, H, gd[t], 4 * H, c[t], c[t + 1], h1[t], H, h2[t][:, H:], 2 * H + 8)
        assert np.allclose(np32(c[t + 1]), c_all[t + 1], rtol=2e-6, atol=2e-6)
        assert_close16(h1[t], h_ref[t], 1e-3, max_ulp=1, what=f"h[{t}]")
        assert np.array_equal(bits(h2[t][:, H:2 * H].contiguous()), bits(h1[t])) and float(h2[t][:, :H].abs().sum()) == 0
    # backward: dh = float(dh_a) + float(dh_b) on the device; the oracle receives that fp32 sum as the gradient from above
    dh_a, dh_b = S16(r.standard_normal((T, B, H))), S16(r.standard_normal((T, B, H)) * 0.3)
    dx_ref, _, _ = L.lstm_layer_bwd(MIXED, dh_a + dh_b, cache, w)      # = dgates of every step (W copies them)
    dcd, dg = torch.zeros(B, H, dtype=torch.float32, device="cuda"), empty16(T, B, 4 * H)
    # the device's own c would do as well; the oracle's keeps this an isolated check of the backward kernel
    for t in (1, 0):
        mp.mp_lstm_cell_bwd(B, H, gd[t], 4 * H, f32(c_all[t]), f32(c_all[t + 1]), h16(dh_a[t]), H, h16(dh_b[t]), H, dcd, dg[t])
        assert_close16(dg[t], dx_ref[t], 1e-3, what=f"dgates[{t}]")
    # one of the two addends may be absent
    dx_ref1, _, _ = L.lstm_layer_bwd(MIXED, dh_a, cache, w)
    dcd.zero_()
    for t in (1, 0):
        mp.mp_lstm_cell_bwd(B, H, gd[t], 4 * H, f32(c_all[t]), f32(c_all[t + 1]), h16(dh_a[t]), H, None, H, dcd, dg[t])
        assert_close16(dg[t], dx_ref1[t], 1e-3, what=f"dgates[{t}] single addend")


def _persistent_lstm_layer(T, Bn, I, H, x_seq, w, b, dh_seq, wait_limit_us=0, extra=0):
    """One LSTM layer through the persistent kernels: input half of the gate sums as one fp32 product, the recurrent
    kernel, and (backward) the recurrent kernel followed by the large input-gradient and weight-gradient products."""
    ld = I + H
    xh = torch.zeros(T, Bn, ld, dtype=torch.float16, device="cuda")
    xh[:, :, :I].copy_(h16(x_seq))
    wd, bd = h16(w), h16(b)
    gx = empty32(T * Bn, 4 * H)
    mp.mp_gemm_fwd(mp.gemm_desc(T * Bn, 4 * H, I, ldx=ld, ldw=ld), xh, wd, None, None, None, gx)
    gates, c = empty16(T, Bn, 4 * H), torch.zeros(T + 1, Bn, H, dtype=torch.float32, device="cuda")
    h_up = torch.full((T, Bn, H + 2), 5.0, dtype=torch.float16, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    ws = torch.zeros(mp.mp_lstm_layer_workspace_bytes() // 4, dtype=torch.int32, device="cuda")
    d = mp.lstm_layer_desc(T, Bn, I, H, ld, ld, H + 2, wait_limit_us, extra)
    mp.mp_lstm_layer_fwd(d, gx, wd, bd, gates, c, xh, h_up, status, ws)
    out = dict(xh=xh, gates=gates, c=c, h_up=h_up, status=status)
    if dh_seq is not None:
        dgates = empty16(T, Bn, 4 * H)
        mp.mp_lstm_layer_bwd(mp.lstm_layer_desc(T, Bn, I, H, ld, ld, H, wait_limit_us, extra), wd, gates, c, h16(dh_seq), dgates, status, ws)
        dx, dw, db = empty16(T * Bn, max(I, 8)), empty16(4 * H, ld), empty16(4 * H)
        if I > 0:
            dx = empty16(T * Bn, I)
            mp.mp_gemm_bwd_dx(mp.gemm_desc(T * Bn, 4 * H, I, ldx=I, ldw=ld), dgates, wd, dx)
        dall = mp.gemm_desc(T * Bn, 4 * H, ld)
        mp.mp_gemm_bwd_dw(dall, dgates, xh, dw, db, None, ws_bytes(mp.mp_gemm_bwd_dw_workspace_bytes(dall, True)))
        out.update(dgates=dgates, dx=dx, dw=dw, db=db)
    return out


@pytest.mark.parametrize("T,Bn,I,H", [(6, 8, 96, 128), (5, 20, 64, 256), (3, 32, 8, 384), (4, 1, 0, 128), (1, 17, 8, 128),
                                      (10, 32, 1024, 1024)])
def test_lstm_persistent_layer_kernels(T, Bn, I, H):
    """All time steps of a layer in one launch per direction against the oracle's layer functions: every stored tensor
    of the forward pass (gate sums, h_t, fp32 cell states) and, from the GPU's own forward tensors, the gradients.
    Shapes: one and several workgroups, batch rows below / between / at the 16-row matrix-core blocks, no input half
    at all (I = 0), and config 5's layer at full width."""
    r = RNG(T * 1000 + Bn + I + H)
    x_seq = S16(r.standard_normal((T, Bn, I)))
    w, b = S16(r.uniform(-0.1, 0.1, (4 * H, I + H))), S16(r.standard_normal(4 * H) * 0.1)
    dh_seq = S16(r.standard_normal((T, Bn, H)))
    h_ref, cache = L.lstm_layer_fwd(MIXED, x_seq, w, b)
    xh_ref, gates_ref, c_ref, _ = cache
    o = _persistent_lstm_layer(T, Bn, I, H, x_seq, w, b, dh_seq)
    assert int(o["status"].item()) == 0
    assert_close16(o["gates"][0], gates_ref[0], 1e-3, max_ulp=1, what="gate sums of step 0")   # same inputs on both sides
    assert_close16(o["gates"], gates_ref, 1e-3, what="gate sums")      # later steps see the device's own h_{t-1}
    assert_close16(o["h_up"][:, :, :H], h_ref, 1e-3, what="h")
    assert torch.all(o["h_up"][:, :, H:] == 5.0)
    assert_close16(o["xh"], xh_ref, 1e-3, what="[x, h_prev] row blocks")
    assert rel_fro(np32(o["c"]), np.stack(c_ref)) <= 1e-3
    # backward from the device's own stored forward tensors (what a training step differentiates)
    cache_gpu = (np32(o["xh"]), np32(o["gates"]), list(np32(o["c"])), I)
    dx_ref, dw_ref, db_ref = L.lstm_layer_bwd(MIXED, dh_seq, cache_gpu, w)
    if I > 0:
        assert_close16(o["dx"].view(T, Bn, I), dx_ref, 1e-3, what="dx")
    assert_close16(o["dw"], dw_ref, 1e-3, what="dW")
    assert_close16(o["db"], db_ref, 1e-3, what="db")


def test_lstm_persistent_layer_timeout_path_and_rejections():
    """The step barrier's wait is bounded: asked to wait for a flag nobody raises (debug_extra_participants) with a
    2 ms limit, every workgroup gives up, the kernels end normally and *status reports it; a poisoned status makes the
    next launch stop at its first barrier; after clearing it the same buffers give the right answer again."""
    T, Bn, I, H = 4, 8, 32, 256
    r = RNG(77)
    x_seq, w, b = S16(r.standard_normal((T, Bn, I))), S16(r.uniform(-0.1, 0.1, (4 * H, I + H))), S16(np.zeros(4 * H))
    o = _persistent_lstm_layer(T, Bn, I, H, x_seq, w, b, S16(r.standard_normal((T, Bn, H))), wait_limit_us=2000, extra=1)
    torch.cuda.synchronize()
    assert int(o["status"].item()) != 0
    h_ref, _ = L.lstm_layer_fwd(MIXED, x_seq, w, b)
    good = _persistent_lstm_layer(T, Bn, I, H, x_seq, w, b, None)
    assert int(good["status"].item()) == 0
    assert_close16(good["h_up"][:, :, :H], h_ref, 1e-3, what="h after a timed-out launch")
    # unsupported shapes are refused before anything is launched
    ws = torch.zeros(mp.mp_lstm_layer_workspace_bytes() // 4, dtype=torch.int32, device="cuda")
    st = torch.zeros(1, dtype=torch.int32, device="cuda")
    for (Bx, Hx, Ix) in ((33, 128, 8), (8, 192, 8), (8, 2048, 8), (8, 128, 4)):
        with pytest.raises(mp.MPError) as e:
            mp.mp_lstm_layer_fwd(mp.lstm_layer_desc(2, Bx, Ix, Hx, Ix + Hx, Ix + Hx, Hx), empty32(2 * Bx, 4 * Hx), empty16(4 * Hx, Ix + Hx),
                                 empty16(4 * Hx), empty16(2, Bx, 4 * Hx), empty32(3, Bx, Hx), empty16(2, Bx, Ix + Hx), None, st, ws)
        assert e.value.code == ML.MP_E_UNSUPPORTED
    with pytest.raises(mp.MPError) as e:
        mp.mp_lstm_layer_fwd(mp.lstm_layer_desc(2, 8, 8, 128, 136, 136, 128), empty32(16, 512), empty16(512, 136), empty16(512),
                             empty16(2, 8, 512), empty32(3, 8, 128), empty16(2, 8, 136), None, None, ws)
    assert e.value.code == ML.MP_E_INVAL


@pytest.mark.parametrize("rows,cols", [(4096, 512), (100, 40), (1, 8), (777, 1001), (8192, 64)])
def test_colsum(rows, cols):
    r = RNG(rows + cols)
    dy = S16(r.standard_normal((rows, cols)))
    db = empty16(cols)
    mp.mp_colsum(rows, cols, h16(dy), cols, db, None, ws_bytes(mp.mp_colsum_workspace_bytes(rows, cols)))
    assert_close16(db, MIXED.store(dy.sum(0, dtype=np.float32)), 1e-3, max_ulp=1, what="colsum")


def test_gradient_producers_flag_their_own_overflow():
    """The column-sum and LayerNorm-backward kernels write fp16 gradients (bias, gamma, beta): when a sum leaves the
    fp16 range the stored value is inf as in the oracle, and the overflow flag of the state they are given is set
    (what MP_UPDATE_PRECHECKED relies on)."""
    rows, cols = 4096, 264
    dy = np.full((rows, cols), 2.0, np.float32)
    dy[:, 5] = 100.0                                           # column 5 sums to 409600: beyond fp16
    dy[:, 9] = -100.0
    ref = MIXED.store(dy.sum(0, dtype=np.float32))
    assert np.isposinf(ref[5]) and np.isneginf(ref[9]) and np.isfinite(np.delete(ref, [5, 9])).all()
    st = make_state()
    db = empty16(cols)
    ws = ws_bytes(mp.mp_colsum_workspace_bytes(rows, cols))
    mp.mp_colsum(rows, cols, h16(dy), cols, db, st, ws)
    assert np.array_equal(bits(db), half_bits(ref)) and mp.scale_state_read(st).found_inf == 1
    st = make_state()
    mp.mp_colsum(rows, cols, h16(np.full((rows, cols), 2.0, np.float32)), cols, db, st, ws)
    assert mp.scale_state_read(st).found_inf == 0 and torch.all(db == 8192.0)
    # a NaN in the input reaches the sum and the flag
    dyn = np.full((rows, cols), 1.0, np.float32)
    dyn[77, 3] = np.nan
    mp.mp_colsum(rows, cols, h16(dyn), cols, db, st, ws)
    assert mp.scale_state_read(st).found_inf == 1 and np.isnan(np32(db)[3]) and np.isfinite(np.delete(np32(db), 3)).all()
    # the weight-gradient entry point with db: flag from the bias gradient alone (dW itself stays finite)
    d = mp.gemm_desc(rows, cols, 64)
    x = np.zeros((rows, 64), np.float32)
    st = make_state()
    dw, db2 = empty16(cols, 64), empty16(cols)
    mp.mp_gemm_bwd_dw(d, h16(dy), h16(x), dw, db2, st, ws_bytes(mp.mp_gemm_bwd_dw_workspace_bytes(d, True)))
    assert torch.all(dw == 0) and np.array_equal(bits(db2), half_bits(ref)) and mp.scale_state_read(st).found_inf == 1

    # LayerNorm backward: dgamma = sum_rows dy xhat, dbeta = sum_rows dy, dz column sums
    rows, d_ = 2048, 256
    r = RNG(5)
    x_, a_ = S16(r.standard_normal((rows, d_))), S16(r.standard_normal((rows, d_)) * 0.5)
    gam = S16(np.ones(d_))
    y_ref, cache = L.layernorm_fwd(MIXED, x_, a_, gam, np.zeros(d_, np.float32))
    xd, ad, gd = h16(x_), h16(a_), h16(gam)
    y, mean, rstd = empty16(rows, d_), empty32(rows), empty32(rows)
    mp.mp_layernorm_fwd(rows, d_, xd, ad, gd, h16(np.zeros(d_)), L.LN_EPS, y, mean, rstd)
    for case in ("dbeta", "dgamma", "clean"):
        dy_ = S16(r.standard_normal((rows, d_)))
        if case == "dbeta":
            dy_[:, 11] = 64.0                                   # 2048 x 64 = 131072 -> inf in dbeta[11]
        elif case == "dgamma":
            dy_[:, 13] = S16(600.0 * np.sign(cache[0][:, 13]))  # sum |xhat| 600 ~ 1e6 -> inf in dgamma[13]
        dz_ref, dg_ref, db_ref = L.layernorm_bwd(MIXED, dy_, cache, gam)
        bad_ref = not (np.isfinite(dg_ref).all() and np.isfinite(db_ref).all()
                       and np.isfinite(MIXED.store(dz_ref.sum(0, dtype=np.float32))).all())
        assert bad_ref == (case != "clean")
        st = make_state()
        dz, dg, dbt, dzs = empty16(rows, d_), empty16(d_), empty16(d_), empty16(d_)
        mp.mp_layernorm_bwd(rows, d_, h16(dy_), xd, ad, gd, mean, rstd, dz, dg, dbt, st,
                            ws_bytes(mp.mp_layernorm_bwd_workspace_bytes(rows, d_)), dz_colsum=dzs)
        assert mp.scale_state_read(st).found_inf == int(bad_ref), case
        assert np.array_equal(np.isfinite(np32(dg)), np.isfinite(dg_ref)) and np.array_equal(np.isfinite(np32(dbt)), np.isfinite(db_ref))


def test_cast_is_rne_and_overflows_to_inf():
    r = RNG(12)
    x = np.concatenate([r.standard_normal(100003).astype(np.float32) * np.float32(s) for s in (1e-7, 1e-3, 1, 7e4)])
    x[:6] = [65520.0, 65519.99, 2.0 ** -25, np.nextafter(np.float32(2.0 ** -25), np.float32(1)), -1e9, np.nan]
    out = empty16(x.size)
    mp.mp_cast_f32_to_f16(x.size, f32(x), out)
    ref = half_bits(MIXED.store(x))
    got = bits(out)
    nan = np.isnan(x)
    assert np.array_equal(got[~nan], ref[~nan]) and np.all((got[nan] & 0x7C00) == 0x7C00)


# ------------------------------------------------------------------ optimizer wrapper and scale policy
def _tensors(r, sizes, adam=True):
    out = []
    for n in sizes:
        out.append(dict(w=r.standard_normal(n).astype(np.float32) * 0.05, g=S16(r.standard_normal(n) * 100),
                        m=r.standard_normal(n).astype(np.float32) * 0.01, v=np.abs(r.standard_normal(n)).astype(np.float32) * 1e-4))
    return out


def _run_update(ts, kind, S, t_prev, wd=0.0, poison=None, flags=0, lr=1e-3):
    host = [dict(g16=t["g"].copy(), w32=t["w"].copy(), w16=MIXED.store(t["w"]), m=t["m"].copy(), v=t["v"].copy()) for t in ts]
    if poison is not None:
        host[poison[0]]["g16"][poison[1]] = poison[2]
    ost = O.ScaleState(scale=S, opt_step=t_prev, growth_interval=3)
    ocfg = I.OptCfg(kind=kind, lr=lr, weight_decay=wd)
    dev = [dict(g16=h16(h["g16"]), w32=f32(h["w32"]), w16=h16(h["w16"]), m=f32(h["m"]), v=f32(h["v"])) for h in host]
    found_ref = O.unscale_check_update(MIXED, host, ocfg, ost)
    O.loss_scale_update(ost, found_ref)
    st = make_state(scale=S, interval=3)
    # bring the device state to the same optimizer step count
    words = st.cpu()
    words[8] = t_prev
    st.copy_(words)
    mp.mp_unscale_check_update(mp.tensor_list(dev), len(dev), mp.opt_cfg(kind, lr, weight_decay=wd), st, flags)
    mp.mp_loss_scale_update(st)
    return host, dev, ost, mp.scale_state_read(st), found_ref


@pytest.mark.parametrize("kind", ["adam", "sgd"])
@pytest.mark.parametrize("t_prev,wd", [(0, 0.0), (1, 1e-4), (57, 1e-2), (3, 0.3)])
def test_update_matches_oracle(kind, t_prev, wd):
    """Unscale + SGD / Adam on the masters + fp16 re-cast, with and without the fp32-side weight decay of Section 3.3
    (g += wd * w32 after unscaling, for both optimizers)."""
    sizes = [8192 * 3 + 5, 1, 7, 4096, 100000, 33] + [64] * 40          # > 32 tensors: several launches
    ts = _tensors(RNG(20 + t_prev), sizes)
    host, dev, ost, dst, found = _run_update(ts, kind, 2.0 ** 7, t_prev, wd=wd)
    assert found == 0 and dst.opt_step == ost.opt_step == t_prev + 1
    for h, d in zip(host, dev):
        assert rel_fro(np32(d["w32"]), h["w32"]) <= 1e-5
        assert np.abs(np32(d["w32"]) - h["w32"]).max() <= 1e-5 * np.abs(h["w32"]).max()
        if kind == "adam":
            assert rel_fro(np32(d["m"]), h["m"]) <= 1e-6 and rel_fro(np32(d["v"]), h["v"]) <= 1e-6
        # the fp16 copy is exactly RNE16 of the master the device holds
        assert np.array_equal(bits(d["w16"]), half_bits(MIXED.store(np32(d["w32"]))))


@pytest.mark.parametrize("bad", [np.inf, -np.inf, np.nan])
@pytest.mark.parametrize("where", [(0, 0), (2, 4095), (5, 32), (45, 63)])
def test_update_skips_on_nonfinite_and_halves_scale(bad, where):
    sizes = [8192 * 3 + 5, 1, 4096, 7, 100000, 33] + [64] * 40
    ts = _tensors(RNG(30), sizes)
    host, dev, ost, dst, found = _run_update(ts, "adam", 2.0 ** 15, 4, poison=(where[0], where[1], bad))
    assert found == 1
    assert (dst.scale, dst.good_steps, dst.opt_step, dst.skipped_steps, dst.found_inf) == (2.0 ** 14, 0, 4, 1, 0)
    assert (ost.scale, ost.good_steps, ost.opt_step, ost.skipped_steps) == (2.0 ** 14, 0, 4, 1)
    assert dst.hist_scale[0] == 2.0 ** 15 and dst.hist_found_inf[0] == 1
    for t, d in zip(ts, dev):                 # every buffer byte-identical to before the call
        assert np.array_equal(np32(d["w32"]).view(np.uint32), t["w"].view(np.uint32))
        assert np.array_equal(np32(d["m"]).view(np.uint32), t["m"].view(np.uint32))
        assert np.array_equal(np32(d["v"]).view(np.uint32), t["v"].view(np.uint32))
        assert np.array_equal(bits(d["w16"]), half_bits(MIXED.store(t["w"])))


def test_update_prechecked_flag_trusts_state():
    ts = _tensors(RNG(31), [5000])
    host, dev, ost, dst, found = _run_update(ts, "sgd", 4.0, 0, poison=(0, 17, np.inf), flags=ML.MP_UPDATE_PRECHECKED)
    # the inspection pass was skipped and nobody had set the flag: the step is applied (inf reaches the master)
    assert found == 1 and dst.opt_step == 1 and not np.isfinite(np32(dev[0]["w32"])[17])


@pytest.mark.parametrize("name", ["c1", "c2", "c4", "c5", "floor"])
def test_scale_policy_sequences(name):
    from test_oracle_optimizer import _golden
    g = _golden()[name]
    st = make_state(scale=g["s0"], interval=g["n"])
    flag = torch.ones(1, dtype=torch.int32, device="cuda")
    for step in range(g["steps"]):
        if step in g["ovf"]:
            st[7:8].copy_(flag)               # found_inf word, as a gradient-producing kernel would set it
        mp.mp_loss_scale_update(st)
    s = mp.scale_state_read(st)
    assert list(s.hist_scale[:g["steps"]]) == g["seq"]
    assert list(s.hist_found_inf[:g["steps"]]) == [int(i in g["ovf"]) for i in range(g["steps"])]
    assert (s.scale, s.good_steps, s.opt_step, s.skipped_steps, s.total_steps) == (g["final"], g["good"], g["t"], g["skipped"], g["steps"])
    assert s.inv_scale == 1.0 / g["final"]


def test_scale_state_static_mode_and_validation():
    st = make_state(mode=ML.MP_SCALE_STATIC, scale=10.0, interval=1)
    flag = torch.ones(1, dtype=torch.int32, device="cuda")
    for f in (0, 1, 0, 0):
        if f:
            st[7:8].copy_(flag)
        mp.mp_loss_scale_update(st)
    s = mp.scale_state_read(st)
    assert s.scale == 10.0 and s.skipped_steps == 1 and s.opt_step == 3 and s.inv_scale == np.float32(1.0) / np.float32(10.0)
    with pytest.raises(mp.MPError):
        mp.mp_scale_state_init(st, 1, 2.0, 0)
    with pytest.raises(mp.MPError):
        mp.mp_scale_state_init(st, 7, 2.0, 1)
