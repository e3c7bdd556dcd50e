"""Layer arithmetic of the oracle (test infrastructure only; plain NumPy).

Every function follows one rule, from Section 3.1 of the paper: contractions
take storage-type operands, accumulate in the arithmetic type (fp32 under the
MIXED policy), and the result of each operation is rounded once to the
storage type (fp16) before the next operation sees it.  Softmax, LayerNorm
statistics, losses and the LSTM cell state are arithmetic-type islands
(Section 3.2 lists such explicitly-fp32 parts).  Activation gradients and
weight gradients are storage-type tensors as well (Section 3.2).

The paper names the models (Transformer, GNMT-style LSTM; Sections 2 and 5.1)
but does not define their layers; the definitions used are the textbook ones
and are stated in each docstring.
"""
from __future__ import annotations

import numpy as np

from .numerics import Policy

LN_EPS = 1e-5


# ---------------------------------------------------------------- linear
def linear_fwd(P: Policy, x, w, b=None, relu=False):
    """Y = act(X W^T + b); X[M,K], W[N,K], b[N].  Section 3.1: fp16 operands,
    accumulate in fp32, bias and activation applied to the accumulator, one
    rounding to storage."""
    acc = x @ w.T
    if b is not None:
        acc = acc + b
    if relu:
        acc = np.maximum(acc, P.scalar(0))
    return P.store(acc)


def linear_bwd(P: Policy, dy, x, w, need_db=True):
    """Gradients of Y = X W^T + b given dY (storage type, already loss-scaled):
    dX = dY W, dW = dY^T X, db = column sums of dY; each accumulated in the
    arithmetic type and rounded once (Section 3.2: gradients are fp16)."""
    dx = P.store(dy @ w)
    dw = P.store(dy.T @ x)
    db = P.store(dy.sum(axis=0, dtype=P.acc)) if need_db else None
    return dx, dw, db


def relu_mask(P: Policy, d_out, out):
    """Gradient through ReLU: zero where the stored activation is not positive."""
    return np.where(out > 0, d_out, P.scalar(0)).astype(P.acc)


def add_store(P: Policy, a, b):
    """Sum of two stored gradient tensors (a residual branch joining), rounded once."""
    return P.store(a + b)


# ---------------------------------------------------------------- LayerNorm
def layernorm_fwd(P: Policy, x, a, gamma, beta, eps=LN_EPS):
    """y = LN(x + a) * gamma + beta over the last axis.  The sum x + a, the mean,
    the (biased) variance and the normalised value stay in the arithmetic
    type; only y is rounded to storage."""
    z = x + a
    n = P.scalar(z.shape[-1])
    mean = z.sum(axis=-1, keepdims=True, dtype=P.acc) / n
    zc = z - mean
    var = (zc * zc).sum(axis=-1, keepdims=True, dtype=P.acc) / n
    rstd = P.scalar(1) / np.sqrt(var + P.scalar(eps))
    xhat = zc * rstd
    y = P.store(xhat * gamma + beta)
    return y, (xhat, rstd)


def layernorm_bwd(P: Policy, dy, cache, gamma):
    """Returns (dz, dgamma, dbeta) with dz the gradient w.r.t. z = x + a, which
    is the gradient of both the residual input and the branch output."""
    xhat, rstd = cache
    n = P.scalar(xhat.shape[-1])
    dxhat = dy * gamma
    m1 = dxhat.sum(axis=-1, keepdims=True, dtype=P.acc) / n
    m2 = (dxhat * xhat).sum(axis=-1, keepdims=True, dtype=P.acc) / n
    dz = P.store(rstd * (dxhat - m1 - xhat * m2))
    dgamma = P.store((dy * xhat).sum(axis=0, dtype=P.acc))
    dbeta = P.store(dy.sum(axis=0, dtype=P.acc))
    return dz, dgamma, dbeta


# ---------------------------------------------------------------- attention
def _heads(t, n_seq, seq_len, n_heads):
    d = t.shape[1]
    return t.reshape(n_seq, seq_len, n_heads, d // n_heads).transpose(0, 2, 1, 3)


def _unheads(t):
    b, h, s, dk = t.shape
    return t.transpose(0, 2, 1, 3).reshape(b * s, h * dk)


def softmax_rows(P: Policy, s):
    """Softmax over the last axis in the arithmetic type, max-subtracted."""
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True, dtype=P.acc)


def attention_fwd(P: Policy, qkv, n_seq, seq_len, n_heads):
    """Scaled dot-product self-attention on a fused projection qkv[T, 3d]
    (columns [0,d) = q, [d,2d) = k, [2d,3d) = v; head h owns columns
    [h*dk, (h+1)*dk) of each).  Per (sequence, head):
      s = store(q k^T / sqrt(dk)),  p = store(softmax(s)),  ctx = store(p v).
    No mask, no dropout."""
    d = qkv.shape[1] // 3
    q = _heads(qkv[:, :d], n_seq, seq_len, n_heads)
    k = _heads(qkv[:, d:2 * d], n_seq, seq_len, n_heads)
    v = _heads(qkv[:, 2 * d:], n_seq, seq_len, n_heads)
    alpha = P.scalar(1.0 / np.sqrt(float(d // n_heads)))
    s = P.store(alpha * (q @ k.transpose(0, 1, 3, 2)))
    p = P.store(softmax_rows(P, s))
    ctx = P.store(p @ v)
    return _unheads(ctx), (q, k, v, p, alpha)


def attention_bwd(P: Policy, dctx, cache):
    """dP = dctx v^T, dV = p^T dctx, dS = p * (dP - rowsum(dP * p)),
    dQ = alpha dS k, dK = alpha dS^T q; each a stored tensor.  Returns dqkv[T,3d]."""
    q, k, v, p, alpha = cache
    b, h, s, dk = q.shape
    dctx_h = _heads(dctx, b, s, h)
    dp = P.store(dctx_h @ v.transpose(0, 1, 3, 2))
    dv = P.store(p.transpose(0, 1, 3, 2) @ dctx_h)
    inner = (dp * p).sum(axis=-1, keepdims=True, dtype=P.acc)
    ds = P.store(p * (dp - inner))
    dq = P.store(alpha * (ds @ k))
    dk_ = P.store(alpha * (ds.transpose(0, 1, 3, 2) @ q))
    return np.concatenate([_unheads(dq), _unheads(dk_), _unheads(dv)], axis=1)


# ---------------------------------------------------------------- losses
def mse_scaled(P: Policy, y, target, scale):
    """L = mean((y - target)^2) (arithmetic type, reported unscaled);
    seed gradient = store(S * 2 (y - target) / numel) (Section 3.1, item 1:
    the loss is scaled so that backpropagated values stay in fp16 range)."""
    diff = y - target
    loss = (diff * diff).sum(dtype=P.acc) / P.scalar(diff.size)
    coef = P.scalar(2.0 * float(scale) / diff.size)
    return loss, P.store(coef * diff)


def softmax_xent_scaled(P: Policy, logits, targets, scale):
    """L = mean over rows of (logsumexp(z) - z[target]), z the stored logits
    brought into the arithmetic type; seed gradient =
    store((S / rows) * (softmax(z) - onehot(target))).  A target outside
    [0, vocab) makes its row contribute zero loss and zero gradient (the mean
    still divides by the number of rows)."""
    rows, vocab = logits.shape
    targets = np.asarray(targets).astype(np.int64)
    valid = (targets >= 0) & (targets < vocab)
    tsafe = np.where(valid, targets, 0)
    zmax = logits.max(axis=-1, keepdims=True)
    e = np.exp(logits - zmax)
    se = e.sum(axis=-1, keepdims=True, dtype=P.acc)
    lse = zmax[:, 0] + np.log(se[:, 0])
    row_loss = np.where(valid, lse - logits[np.arange(rows), tsafe], P.scalar(0))
    loss = row_loss.sum(dtype=P.acc) / P.scalar(rows)
    g = e / se
    g[np.arange(rows), tsafe] -= np.where(valid, P.scalar(1), P.scalar(0))
    g = np.where(valid[:, None], g, P.scalar(0))
    coef = P.scalar(float(scale) / rows)
    return loss, P.store(coef * g)


# ---------------------------------------------------------------- LSTM
def _sigmoid(P: Policy, x):
    return P.scalar(1) / (P.scalar(1) + np.exp(-x))


def lstm_layer_fwd(P: Policy, x_seq, w, b):
    """Plain LSTM cell unrolled over time: x_seq[T,B,I], W[4H, I+H], b[4H].
      gates_t = store([x_t, h_{t-1}] W^T + b), row blocks ordered (i, f, g, o)
      c_t = sigma(f) c_{t-1} + sigma(i) tanh(g)      (arithmetic type, never rounded)
      h_t = store(sigma(o) tanh(c_t)),   h_0 = c_0 = 0.
    No peepholes, projection or forget-gate offset."""
    T, B, _ = x_seq.shape
    H = w.shape[0] // 4
    h = np.zeros((B, H), dtype=P.acc)
    c = np.zeros((B, H), dtype=P.acc)
    xh_all, gates_all, c_all, h_all = [], [], [c], []
    for t in range(T):
        xh = np.concatenate([x_seq[t], h], axis=1)
        gates = P.store(xh @ w.T + b)
        gi, gf, gg, go = (gates[:, j * H:(j + 1) * H] for j in range(4))
        c = _sigmoid(P, gf) * c + _sigmoid(P, gi) * np.tanh(gg)
        h = P.store(_sigmoid(P, go) * np.tanh(c))
        xh_all.append(xh); gates_all.append(gates); c_all.append(c); h_all.append(h)
    return np.stack(h_all), (np.stack(xh_all), np.stack(gates_all), c_all, x_seq.shape[2])


def lstm_layer_bwd(P: Policy, dh_seq, cache, w):
    """Back-propagation through time.  Per step (t descending), with dh the
    arithmetic-type sum of the gradient from the layer above and the recurrent
    gradient, and dc carried in the arithmetic type:
      do = dh tanh(c_t) s_o(1-s_o);  dc += dh s_o (1 - tanh(c_t)^2)
      di = dc tanh(g) s_i(1-s_i);  df = dc c_{t-1} s_f(1-s_f);  dg = dc s_i (1 - tanh(g)^2)
      dgates_t = store([di, df, dg, do]);  [dx_t, dh_{t-1}] = store(dgates_t W);  dc <- dc s_f
    dW = store(sum over all (t, batch) rows of dgates^T [x, h]); db likewise."""
    xh_all, gates_all, c_all, I = cache
    T, B, _ = xh_all.shape
    H = w.shape[0] // 4
    one = P.scalar(1)
    dh_rec = np.zeros((B, H), dtype=P.acc)
    dc = np.zeros((B, H), dtype=P.acc)
    dx_seq = np.zeros((T, B, I), dtype=P.acc)
    dgates_all = np.zeros((T, B, 4 * H), dtype=P.acc)
    for t in range(T - 1, -1, -1):
        gates = gates_all[t]
        gi, gf, gg, go = (gates[:, j * H:(j + 1) * H] for j in range(4))
        si, sf, so = _sigmoid(P, gi), _sigmoid(P, gf), _sigmoid(P, go)
        tg, tc = np.tanh(gg), np.tanh(c_all[t + 1])
        dh = dh_seq[t] + dh_rec
        d_o = dh * tc * so * (one - so)
        dc = dc + dh * so * (one - tc * tc)
        d_i = dc * tg * si * (one - si)
        d_f = dc * c_all[t] * sf * (one - sf)
        d_g = dc * si * (one - tg * tg)
        dc = dc * sf
        dgates = P.store(np.concatenate([d_i, d_f, d_g, d_o], axis=1))
        dgates_all[t] = dgates
        dxh = P.store(dgates @ w)
        dx_seq[t] = dxh[:, :I]
        dh_rec = dxh[:, I:]
    dg2 = dgates_all.reshape(T * B, 4 * H)
    dw = P.store(dg2.T @ xh_all.reshape(T * B, -1))
    db = P.store(dg2.sum(axis=0, dtype=P.acc))
    return dx_seq, dw, db
