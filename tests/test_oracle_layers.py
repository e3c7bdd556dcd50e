"""Pins for the oracle's layer maths: finite differences and library/textbook
routines in fp64 storage, closed forms, invariants (CPU only)."""
import math

import numpy as np
import pytest
import torch

import mp_inputs as I
from oracle import MIXED, FP32, FP64
from oracle import layers as L
from oracle import models as Mo


def _rel(a, b):
    return float(np.linalg.norm(np.asarray(a, np.float64) - np.asarray(b, np.float64)) /
                 max(np.linalg.norm(np.asarray(b, np.float64)), 1e-300))


def _fd_check(fwd_bwd, w, batch, n_probe=6, h=1e-6, tol=2e-6, seed=0):
    """Central differences of the fp64 loss against every returned gradient (scale 1)."""
    rng = np.random.default_rng(seed)
    loss, grads = fwd_bwd(FP64, w, batch, 1.0)
    assert set(grads) == set(w)
    for name, g in grads.items():
        assert g.shape == w[name].shape
        flat = w[name].reshape(-1)
        for idx in rng.choice(flat.size, size=min(n_probe, flat.size), replace=False):
            old = flat[idx]
            flat[idx] = old + h
            lp, _ = fwd_bwd(FP64, w, batch, 1.0)
            flat[idx] = old - h
            lm, _ = fwd_bwd(FP64, w, batch, 1.0)
            flat[idx] = old
            fd = (lp - lm) / (2 * h)
            an = g.reshape(-1)[idx]
            assert abs(fd - an) <= tol * max(1.0, abs(fd), abs(an)) or abs(fd - an) <= 1e-9, (name, idx, fd, an)


def _f64(d):
    return {k: (np.asarray(v, np.float64) if not np.issubdtype(np.asarray(v).dtype, np.integer) else v)
            for k, v in d.items()}


# ----------------------------------------------------------------- finite differences
def test_fd_mlp():
    wl = I.MLPWorkload(rows=5, d_in=7, d_hidden=11, d_out=3)
    w = _f64(wl.masters())
    w["b1"] += 0.1
    w["b2"] -= 0.2
    _fd_check(Mo.mlp_fwd_bwd, w, _f64(wl.batch()))


def test_fd_transformer_two_layers():
    wl = I.TransformerWorkload(index=2, n_layers=2, d_model=8, n_heads=2, d_ff=12, seq_len=4, n_seq=3)
    w = _f64(Mo.flatten_layers(wl.masters()))
    rng = np.random.default_rng(5)
    for k in w:                                   # make biases / LN affine non-trivial
        if w[k].ndim == 1:
            w[k] = w[k] + 0.3 * rng.standard_normal(w[k].shape)
    f = Mo.make_transformer_fwd_bwd(wl.n_layers, wl.n_seq, wl.seq_len, wl.n_heads)
    _fd_check(f, w, _f64(wl.batch()), n_probe=4)


def test_fd_xent_head():
    wl = I.XentWorkload(tokens=6, d_model=5, vocab=9)
    w = _f64(wl.masters())
    w["b"] += 0.1 * np.random.default_rng(6).standard_normal(9)
    _fd_check(Mo.xent_head_fwd_bwd, w, _f64(wl.batch()))


def test_fd_lstm_two_layers():
    wl = I.LSTMWorkload(n_layers=2, hidden=4, d_in=3, batch_size=2, seq_len=3)
    w = _f64(Mo.flatten_layers(wl.masters()))
    for k in w:
        w[k] = w[k] * 5 + (0.2 if w[k].ndim == 1 else 0.0)
    _fd_check(Mo.make_lstm_fwd_bwd(2), w, _f64(wl.batch()))


# ----------------------------------------------------------------- library routines (fp64)
def test_encoder_layer_matches_torch_autograd():
    d, h, ff, S, B = 16, 4, 24, 5, 3
    wl = I.TransformerWorkload(index=2, n_layers=1, d_model=d, n_heads=h, d_ff=ff, seq_len=S, n_seq=B)
    w = _f64(Mo.flatten_layers(wl.masters()))
    rng = np.random.default_rng(7)
    for k in w:
        if w[k].ndim == 1:
            w[k] = w[k] + 0.3 * rng.standard_normal(w[k].shape)
    batch = _f64(wl.batch())
    loss, grads = Mo.make_transformer_fwd_bwd(1, B, S, h)(FP64, w, batch, 1.0)

    tl = torch.nn.TransformerEncoderLayer(d, h, ff, dropout=0.0, activation="relu", batch_first=True,
                                          norm_first=False, layer_norm_eps=L.LN_EPS).double()
    names = {"self_attn.in_proj_weight": "wqkv", "self_attn.in_proj_bias": "bqkv",
             "self_attn.out_proj.weight": "wo", "self_attn.out_proj.bias": "bo",
             "norm1.weight": "ln1_g", "norm1.bias": "ln1_b", "linear1.weight": "w1", "linear1.bias": "b1",
             "linear2.weight": "w2", "linear2.bias": "b2", "norm2.weight": "ln2_g", "norm2.bias": "ln2_b"}
    with torch.no_grad():
        for tn, on in names.items():
            dict(tl.named_parameters())[tn].copy_(torch.from_numpy(w["l0." + on]))
    tl.train()
    x = torch.from_numpy(batch["x"]).reshape(B, S, d)
    y = tl(x).reshape(B * S, d)
    tloss = torch.mean((y - torch.from_numpy(batch["target"])) ** 2)
    tloss.backward()
    assert abs(float(tloss.detach()) - float(loss)) < 1e-12 * max(1, abs(float(loss)))
    for tn, on in names.items():
        assert _rel(grads["l0." + on], dict(tl.named_parameters())[tn].grad.numpy()) < 1e-10, on


def test_lstm_matches_torch_autograd():
    wl = I.LSTMWorkload(n_layers=2, hidden=6, d_in=5, batch_size=3, seq_len=4)
    w = _f64(Mo.flatten_layers(wl.masters()))
    for k in w:
        w[k] = w[k] * 4 + (0.1 if w[k].ndim == 1 else 0.0)
    batch = _f64(wl.batch())
    loss, grads = Mo.make_lstm_fwd_bwd(2)(FP64, w, batch, 1.0)
    tl = torch.nn.LSTM(5, 6, num_layers=2).double()       # gate order i, f, g, o like the oracle
    with torch.no_grad():
        for l in range(2):
            i_dim = 5 if l == 0 else 6
            W = torch.from_numpy(w[f"l{l}.w"])
            getattr(tl, f"weight_ih_l{l}").copy_(W[:, :i_dim])
            getattr(tl, f"weight_hh_l{l}").copy_(W[:, i_dim:])
            getattr(tl, f"bias_ih_l{l}").copy_(torch.from_numpy(w[f"l{l}.b"]))
            getattr(tl, f"bias_hh_l{l}").zero_()
    out, _ = tl(torch.from_numpy(batch["x"]))
    tloss = torch.mean((out - torch.from_numpy(batch["target"])) ** 2)
    tloss.backward()
    assert abs(float(tloss.detach()) - float(loss)) < 1e-12
    for l in range(2):
        i_dim = 5 if l == 0 else 6
        gw = torch.cat([getattr(tl, f"weight_ih_l{l}").grad, getattr(tl, f"weight_hh_l{l}").grad], dim=1).numpy()
        assert _rel(grads[f"l{l}.w"], gw) < 1e-10
        assert _rel(grads[f"l{l}.b"], getattr(tl, f"bias_ih_l{l}").grad.numpy()) < 1e-10


def test_xent_matches_torch_cross_entropy():
    rng = np.random.default_rng(8)
    z = rng.standard_normal((7, 13)) * 3
    t = rng.integers(0, 13, size=7)
    loss, g = L.softmax_xent_scaled(FP64, z, t, 8.0)
    zt = torch.from_numpy(z).requires_grad_()
    tl = torch.nn.functional.cross_entropy(zt, torch.from_numpy(t), reduction="mean")
    tl.backward()
    assert abs(float(loss) - float(tl)) < 1e-13
    assert _rel(g, 8.0 * zt.grad.numpy()) < 1e-13


# ----------------------------------------------------------------- closed forms and invariants
def test_mse_closed_form():
    rng = np.random.default_rng(9)
    y, t = rng.standard_normal((4, 6)), rng.standard_normal((4, 6))
    loss, dy = L.mse_scaled(FP64, y, t, 4.0)
    assert abs(loss - np.mean((y - t) ** 2)) < 1e-15
    assert np.allclose(dy, 4.0 * 2 * (y - t) / 24, rtol=1e-15)
    l0, d0 = L.mse_scaled(MIXED, MIXED.store(y), MIXED.store(y), 1024.0)
    assert l0 == 0 and not d0.any()


def test_xent_closed_forms():
    V = 32768
    z = np.zeros((3, V), dtype=np.float32)
    t = np.array([0, 17, V - 1])
    loss, g = L.softmax_xent_scaled(MIXED, z, t, 2.0 ** 15)
    assert abs(float(loss) - 15 * math.log(2.0)) < 1e-5          # ln 32768 = 10.39720770839918
    assert abs(15 * math.log(2.0) - 10.39720770839918) < 1e-14
    # gradient = (S/rows)(p - onehot): off-target entries S/(rows V) = 1/3, target entry 1/3 - S/3
    assert np.allclose(g[0, 1], np.float16(1 / 3)) and np.allclose(g[0, 0], np.float16(1 / 3 - 2.0 ** 15 / 3), rtol=1e-3)
    z2 = np.zeros((2, 50))
    z2[0, 3] = 200.0
    z2[1, 9] = 200.0
    loss2, g2 = L.softmax_xent_scaled(FP64, z2, np.array([3, 9]), 1.0)
    assert loss2 < 1e-80 and np.abs(g2).max() < 1e-80
    rng = np.random.default_rng(10)
    z3 = rng.standard_normal((11, 40)) * 4
    _, g3 = L.softmax_xent_scaled(FP64, z3, rng.integers(0, 40, 11), 3.0)
    assert np.abs(g3.sum(axis=1)).max() < 1e-15                   # rows of p - onehot sum to zero
    # shift invariance and stability with huge logits
    l_a, _ = L.softmax_xent_scaled(FP64, z3 + 1000.0, np.zeros(11, int), 1.0)
    l_b, _ = L.softmax_xent_scaled(FP64, z3, np.zeros(11, int), 1.0)
    assert abs(l_a - l_b) < 1e-10


def test_xent_out_of_range_target_contributes_nothing():
    rng = np.random.default_rng(11)
    z = rng.standard_normal((4, 10))
    t = np.array([2, -1, 10, 5])
    loss, g = L.softmax_xent_scaled(FP64, z, t, 1.0)
    la, ga = L.softmax_xent_scaled(FP64, z[[0, 3]], t[[0, 3]], 1.0)
    assert abs(loss - la * 2 / 4) < 1e-15
    assert not g[1].any() and not g[2].any()
    assert np.allclose(g[[0, 3]], ga * 2 / 4)


def test_layernorm_invariants():
    rng = np.random.default_rng(12)
    x, a = rng.standard_normal((6, 32)), rng.standard_normal((6, 32))
    g, b = np.ones(32), np.zeros(32)
    y, cache = L.layernorm_fwd(FP64, x, a, g, b)
    assert np.abs(y.mean(axis=1)).max() < 1e-14
    assert np.abs((y * y).mean(axis=1) - 1).max() < 1e-4           # var/(var+eps)
    ty = torch.nn.functional.layer_norm(torch.from_numpy(x + a), (32,), eps=L.LN_EPS).numpy()
    assert np.allclose(y, ty, atol=1e-13)
    dy = rng.standard_normal((6, 32))
    dz, dg, db = L.layernorm_bwd(FP64, dy, cache, g)
    xhat = cache[0]
    assert np.abs(dz.sum(axis=1)).max() < 1e-13                    # dz rows sum to zero
    # ... and are orthogonal to xhat up to the eps in the variance: sum(xhat^2) = n var/(var+eps)
    assert np.abs((dz * xhat).sum(axis=1)).max() < 20 * L.LN_EPS
    assert np.allclose(db, dy.sum(0)) and np.allclose(dg, (dy * xhat).sum(0))


def test_attention_matches_sdpa_and_rows_of_p_sum_to_one():
    rng = np.random.default_rng(13)
    B, S, h, dk = 2, 5, 3, 4
    qkv = rng.standard_normal((B * S, 3 * h * dk))
    ctx, (q, k, v, p, alpha) = L.attention_fwd(FP64, qkv, B, S, h)
    assert np.abs(p.sum(-1) - 1).max() < 1e-14
    tq, tk, tv = (torch.from_numpy(np.ascontiguousarray(t)) for t in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).numpy()
    assert np.allclose(ctx, ref.transpose(0, 2, 1, 3).reshape(B * S, h * dk), atol=1e-13)


def test_mixed_tracks_fp64_within_half_precision():
    wl = I.C2_SMALL
    w32 = Mo.flatten_layers(wl.masters())
    f = Mo.make_transformer_fwd_bwd(wl.n_layers, wl.n_seq, wl.seq_len, wl.n_heads)
    wm = {k: MIXED.store(v) for k, v in w32.items()}
    bm = Mo.island_batch(MIXED, wl.batch())
    S = 2.0 ** 12
    lm, gm = f(MIXED, wm, bm, S)
    l64, g64 = f(FP64, _f64(wm), _f64(bm), S)
    assert abs(lm - l64) / l64 < 1e-3
    for k in gm:
        if gm[k].ndim == 2:
            assert _rel(gm[k], g64[k]) < 4e-3, k


# ----------------------------------------------------------------- where the fp16 roundings sit under MIXED
class _Spy:
    """MIXED with a record of every rounding to storage: (shape, values before rounding were all representable?)."""

    def __init__(self):
        self.log = []
        self.name, self.acc, self.half_storage = MIXED.name, MIXED.acc, MIXED.half_storage

    def island(self, x):
        return MIXED.island(x)

    def scalar(self, v):
        return MIXED.scalar(v)

    def store(self, x):
        y = MIXED.store(x)
        self.log.append((tuple(np.shape(x)), bool(np.array_equal(np.asarray(x, np.float32), y))))
        return y

    def shapes(self):
        out, self.log = [s for s, _ in self.log], []
        return out


def _representable(x):
    return bool(np.array_equal(MIXED.store(x), np.asarray(x, np.float32)))


def test_mixed_storage_points_of_attention_layernorm_and_lstm():
    """Sections 3.1 / 3.2: activations, activation gradients and weight gradients are fp16 tensors; softmax, LayerNorm
    statistics, the loss value and the LSTM cell state are fp32 islands.  The finite-difference and autograd pins run
    in FP64 mode, where a rounding to storage is the identity, so they cannot see a rounding that is missing or
    misplaced under MIXED.  This pin can: it records every rounding each function performs (a dropped, added or moved
    one changes the list) and checks that what is handed on is fp16-representable exactly where a tensor is stored and
    is NOT where it is an fp32 island."""
    rng = np.random.default_rng(7)
    P = _Spy()
    # ---- attention: scores, probabilities, context | dP, dV, dS, dQ, dK
    B, S, H, dk = 2, 5, 3, 4
    d = H * dk
    qkv = MIXED.store(rng.standard_normal((B * S, 3 * d)))
    ctx, cache = L.attention_fwd(P, qkv, B, S, H)
    assert P.shapes() == [(B, H, S, S), (B, H, S, S), (B, H, S, dk)]
    q, k, v, p, alpha = cache
    assert all(_representable(t) for t in (ctx, p)) and ctx.dtype == np.float32
    assert alpha == np.float32(0.5)                                   # 1/sqrt(dk), applied to the fp32 sum before rounding
    dqkv = L.attention_bwd(P, MIXED.store(rng.standard_normal((B * S, d))), cache)
    assert P.shapes() == [(B, H, S, S), (B, H, S, dk), (B, H, S, S), (B, H, S, dk), (B, H, S, dk)]
    assert _representable(dqkv) and dqkv.shape == (B * S, 3 * d)
    # the softmax island: probabilities are rounded once, from fp32 values that were not representable
    P.store(L.softmax_rows(P, MIXED.store(rng.standard_normal((3, 7)))))
    assert P.log[-1] == ((3, 7), False)
    P.shapes()
    # ---- LayerNorm: only y is stored forward (sum x + a, statistics, xhat stay fp32); dz, dgamma, dbeta backward
    T = 6
    x, a = MIXED.store(rng.standard_normal((T, d))), MIXED.store(rng.standard_normal((T, d)))
    gam, bet = MIXED.store(1 + 0.1 * rng.standard_normal(d)), MIXED.store(0.1 * rng.standard_normal(d))
    y, (xhat, rstd) = L.layernorm_fwd(P, x, a, gam, bet)
    assert P.shapes() == [(T, d)]
    assert _representable(y) and not _representable(xhat) and not _representable(rstd)
    # the residual sum is not rounded before the statistics: x + a with a 1-ulp-of-x tail must still move the mean
    big, tail = np.full((1, d), 2048.0, np.float32), np.zeros((1, d), np.float32)
    tail[0, 0] = 1.0                                                  # 2049 is not an fp16 value
    _, (xh1, _) = L.layernorm_fwd(MIXED, big, tail, np.ones(d, np.float32), np.zeros(d, np.float32))
    assert xh1[0, 0] > 1.0                                            # rounded to 2048 it would be a constant row: xhat = 0
    dz, dg, db = L.layernorm_bwd(P, MIXED.store(rng.standard_normal((T, d))), (xhat, rstd), gam)
    assert P.shapes() == [(T, d), (d,), (d,)]
    assert all(_representable(t) for t in (dz, dg, db))
    # ---- LSTM: gates and h are stored every step, c never; backward: dgates and [dx, dh] every step, then dW, db
    Tn, Bn, I_, Hn = 3, 2, 5, 4
    w, b = MIXED.store(rng.standard_normal((4 * Hn, I_ + Hn)) * 0.5), MIXED.store(rng.standard_normal(4 * Hn) * 0.1)
    h_seq, lc = L.lstm_layer_fwd(P, MIXED.store(rng.standard_normal((Tn, Bn, I_))), w, b)
    assert P.shapes() == [(Bn, 4 * Hn), (Bn, Hn)] * Tn
    xh_all, gates_all, c_all, _ = lc
    assert _representable(h_seq) and _representable(gates_all) and _representable(xh_all)
    assert all(not _representable(c) for c in c_all[1:])            # the cell state is carried in fp32
    dx, dw, db = L.lstm_layer_bwd(P, MIXED.store(rng.standard_normal((Tn, Bn, Hn))), lc, w)
    assert P.shapes() == [(Bn, 4 * Hn), (Bn, I_ + Hn)] * Tn + [(4 * Hn, I_ + Hn), (4 * Hn,)]
    assert all(_representable(t) for t in (dx, dw, db))
    # ---- linear, losses, the join of two gradient branches
    xx, ww, bb = MIXED.store(rng.standard_normal((T, d))), MIXED.store(rng.standard_normal((7, d))), MIXED.store(rng.standard_normal(7))
    yy = L.linear_fwd(P, xx, ww, bb, relu=True)
    assert P.shapes() == [(T, 7)]                                     # bias and ReLU act on the fp32 sum: ONE rounding
    L.linear_bwd(P, MIXED.store(rng.standard_normal((T, 7))), xx, ww)
    assert P.shapes() == [(T, d), (7, d), (7,)]
    loss, dy = L.mse_scaled(P, yy, MIXED.store(rng.standard_normal((T, 7))), 1024.0)
    assert P.shapes() == [(T, 7)] and not _representable(loss) and _representable(dy)
    loss, dz_ = L.softmax_xent_scaled(P, yy, rng.integers(0, 7, T), 1024.0)
    assert P.shapes() == [(T, 7)] and _representable(dz_)
    L.add_store(P, yy, yy)
    assert P.shapes() == [(T, 7)]


def test_mixed_encoder_layer_roundings_in_order():
    """The whole encoder layer under MIXED: forward stores qkv, scores, p, ctx, attention output, y1, f, g, y2 (9);
    backward stores, in the order of the chain rule, the three LayerNorm-2 gradients, the FFN gradients with the
    residual join, the three LayerNorm-1 gradients, the projection gradients, the five attention gradients, the
    fused-projection gradients and the join into dx (24)."""
    wl = I.TransformerWorkload(index=2, n_layers=1, d_model=8, n_heads=2, d_ff=12, seq_len=4, n_seq=3)
    P = _Spy()
    w = {k: MIXED.store(v) for k, v in Mo.flatten_layers(wl.masters()).items()}
    T, d, f, B, S, H = wl.tokens, 8, 12, 3, 4, 2
    y2, c = Mo.encoder_layer_fwd(P, w, "l0.", MIXED.store(wl.batch()["x"]), B, S, H)
    att = [(B, H, S, S), (B, H, S, S), (B, H, S, d // H)]
    assert P.shapes() == [(T, 3 * d)] + att + [(T, d), (T, d), (T, f), (T, d), (T, d)]
    grads = {}
    Mo.encoder_layer_bwd(P, w, "l0.", MIXED.store(wl.batch()["target"] * 0.01), c, grads)
    hd = (B, H, S, d // H)
    assert P.shapes() == ([(T, d), (d,), (d,)]                       # LN2: dz2, dgamma, dbeta
                          + [(T, f), (d, f), (d,)]                   # W2: df, dW2, db2   (the ReLU mask is a select: no rounding)
                          + [(T, d), (f, d), (f,)] + [(T, d)]        # W1: dy1 branch, dW1, db1; join with dz2
                          + [(T, d), (d,), (d,)]                     # LN1
                          + [(T, d), (d, d), (d,)]                   # Wo: dctx, dWo, dbo
                          + [(B, H, S, S), hd, (B, H, S, S), hd, hd] # attention: dP, dV, dS, dQ, dK
                          + [(T, d), (3 * d, d), (3 * d,)] + [(T, d)])  # Wqkv: dx branch, dW, db; join with dz1
    assert set(grads) == set(w) and all(_representable(g) for g in grads.values())
