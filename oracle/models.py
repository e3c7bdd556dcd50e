"""Forward/backward of the five workloads and the training loop (oracle; test
infrastructure only).

Each `*_fwd_bwd(P, w, batch, scale)` takes stored (fp16-representable under
MIXED) weights `w` as a flat dict name -> array, runs forward, the loss, and
the loss-scaled backward pass, and returns (loss, grads) with grads a flat dict
of stored gradients under the same names.  `train` strings these steps
together with the optimizer wrapper and the scale policy in the order the
paper gives (Sections 3.1 and 3.2): forward and backward on the fp16 copies
with the current scale, inspect gradients, update masters or skip, set the
next scale.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional

import numpy as np

from . import layers as L
from .numerics import Policy
from .optimizer import ScaleState, loss_scale_update, unscale_check_update


def flatten_layers(per_layer: List[Dict[str, np.ndarray]]) -> Dict[str, np.ndarray]:
    return {f"l{i}.{k}": v for i, lay in enumerate(per_layer) for k, v in lay.items()}


# ------------------------------------------------------------------ config 1
def mlp_fwd_bwd(P: Policy, w, batch, scale, keep=None):
    x, target = batch["x"], batch["target"]
    h = L.linear_fwd(P, x, w["w1"], w["b1"], relu=True)
    y = L.linear_fwd(P, h, w["w2"], w["b2"])
    loss, dy = L.mse_scaled(P, y, target, scale)
    dh, dw2, db2 = L.linear_bwd(P, dy, h, w["w2"])
    dpre = L.relu_mask(P, dh, h)
    dx, dw1, db1 = L.linear_bwd(P, dpre, x, w["w1"])
    if keep is not None:
        keep.update(h=h, y=y, dy=dy, dpre=dpre, dx=dx)
    return loss, {"w1": dw1, "b1": db1, "w2": dw2, "b2": db2}


# ------------------------------------------------------------- configs 2, 3
def encoder_layer_fwd(P: Policy, w, pre, x, n_seq, seq_len, n_heads):
    """Post-LayerNorm Transformer encoder layer:
    y1 = LN(x + Wo attention(Wqkv x)),  y2 = LN(y1 + W2 relu(W1 y1))."""
    qkv = L.linear_fwd(P, x, w[pre + "wqkv"], w[pre + "bqkv"])
    ctx, att = L.attention_fwd(P, qkv, n_seq, seq_len, n_heads)
    a = L.linear_fwd(P, ctx, w[pre + "wo"], w[pre + "bo"])
    y1, ln1 = L.layernorm_fwd(P, x, a, w[pre + "ln1_g"], w[pre + "ln1_b"])
    f = L.linear_fwd(P, y1, w[pre + "w1"], w[pre + "b1"], relu=True)
    g = L.linear_fwd(P, f, w[pre + "w2"], w[pre + "b2"])
    y2, ln2 = L.layernorm_fwd(P, y1, g, w[pre + "ln2_g"], w[pre + "ln2_b"])
    return y2, dict(x=x, qkv=qkv, ctx=ctx, att=att, a=a, y1=y1, ln1=ln1, f=f, g=g, ln2=ln2)


def encoder_layer_bwd(P: Policy, w, pre, dy2, c, grads):
    dz2, grads[pre + "ln2_g"], grads[pre + "ln2_b"] = L.layernorm_bwd(P, dy2, c["ln2"], w[pre + "ln2_g"])
    df, grads[pre + "w2"], grads[pre + "b2"] = L.linear_bwd(P, dz2, c["f"], w[pre + "w2"])
    dpre = L.relu_mask(P, df, c["f"])
    dy1_ffn, grads[pre + "w1"], grads[pre + "b1"] = L.linear_bwd(P, dpre, c["y1"], w[pre + "w1"])
    dy1 = L.add_store(P, dy1_ffn, dz2)
    dz1, grads[pre + "ln1_g"], grads[pre + "ln1_b"] = L.layernorm_bwd(P, dy1, c["ln1"], w[pre + "ln1_g"])
    dctx, grads[pre + "wo"], grads[pre + "bo"] = L.linear_bwd(P, dz1, c["ctx"], w[pre + "wo"])
    dqkv = L.attention_bwd(P, dctx, c["att"])
    dx_att, grads[pre + "wqkv"], grads[pre + "bqkv"] = L.linear_bwd(P, dqkv, c["x"], w[pre + "wqkv"])
    return L.add_store(P, dx_att, dz1)


def make_transformer_fwd_bwd(n_layers, n_seq, seq_len, n_heads):
    def fwd_bwd(P: Policy, w, batch, scale, keep=None):
        h, caches = batch["x"], []
        for l in range(n_layers):
            h, c = encoder_layer_fwd(P, w, f"l{l}.", h, n_seq, seq_len, n_heads)
            caches.append(c)
        loss, dh = L.mse_scaled(P, h, batch["target"], scale)
        grads = {}
        if keep is not None:
            keep.update(y=h, dy=dh, caches=caches)
        for l in range(n_layers - 1, -1, -1):
            dh = encoder_layer_bwd(P, w, f"l{l}.", dh, caches[l], grads)
        if keep is not None:
            keep["dx"] = dh
        return loss, grads
    return fwd_bwd


# ------------------------------------------------------------------ config 4
def xent_head_fwd_bwd(P: Policy, w, batch, scale, keep=None):
    h, targets = batch["h"], batch["targets"]
    logits = L.linear_fwd(P, h, w["w"], w["b"])
    loss, dlogits = L.softmax_xent_scaled(P, logits, targets, scale)
    dh, dw, db = L.linear_bwd(P, dlogits, h, w["w"])
    if keep is not None:
        keep.update(logits=logits, dlogits=dlogits, dh=dh)
    return loss, {"w": dw, "b": db}


# ------------------------------------------------------------------ config 5
def make_lstm_fwd_bwd(n_layers):
    def fwd_bwd(P: Policy, w, batch, scale, keep=None):
        seq, caches = batch["x"], []
        for l in range(n_layers):
            seq, c = L.lstm_layer_fwd(P, seq, w[f"l{l}.w"], w[f"l{l}.b"])
            caches.append(c)
        loss, dseq = L.mse_scaled(P, seq, batch["target"], scale)
        if keep is not None:
            keep.update(y=seq, dy=dseq)
        grads = {}
        for l in range(n_layers - 1, -1, -1):
            dseq, grads[f"l{l}.w"], grads[f"l{l}.b"] = L.lstm_layer_bwd(P, dseq, caches[l], w[f"l{l}.w"])
        if keep is not None:
            keep["dx"] = dseq
        return loss, grads
    return fwd_bwd


# ------------------------------------------------------------------ training
class Trainer:
    """Masters, stored copies, optimizer moments and scale state of one model."""

    def __init__(self, P: Policy, masters: Dict[str, np.ndarray], opt, scale_cfg):
        self.P, self.opt = P, opt
        self.names = list(masters)
        self.w32 = {k: P.island(v).copy() for k, v in masters.items()}
        self.w16 = {k: P.store(v) for k, v in self.w32.items()}
        self.m = {k: np.zeros_like(v) for k, v in self.w32.items()}
        self.v = {k: np.zeros_like(v) for k, v in self.w32.items()}
        self.state = ScaleState(mode=scale_cfg.mode, scale=float(scale_cfg.init_scale),
                                growth_interval=scale_cfg.growth_interval,
                                min_scale=float(scale_cfg.min_scale), max_scale=float(scale_cfg.max_scale))
        self.losses: List[float] = []

    def apply(self, grads: Dict[str, np.ndarray]) -> int:
        """Optimizer wrapper + scale policy for one set of stored gradients."""
        tensors = [dict(g16=grads[k], w32=self.w32[k], w16=self.w16[k], m=self.m[k], v=self.v[k])
                   for k in self.names]
        found = unscale_check_update(self.P, tensors, self.opt, self.state)
        loss_scale_update(self.state, found)
        return found

    def step(self, fwd_bwd: Callable, batch, inject: Optional[Callable] = None) -> Dict[str, np.ndarray]:
        loss, grads = fwd_bwd(self.P, self.w16, batch, self.state.scale)
        if inject is not None:
            inject(grads)
        self.losses.append(float(loss))
        self.apply(grads)
        return grads


def island_batch(P: Policy, batch: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
    """Inputs and regression targets enter the model as stored (fp16) tensors;
    integer class targets pass through."""
    return {k: (v if np.issubdtype(np.asarray(v).dtype, np.integer) else P.store(v)) for k, v in batch.items()}
