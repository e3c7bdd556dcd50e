"""Seeded synthetic inputs for the five mixed-precision training workloads.

This module only draws random numbers and names shapes.  It holds none of the
method's arithmetic (no fp16 rounding, no layer maths, no optimizer): both the
CPU oracle's tests and the HIP path's tests/bench take the fp32 arrays drawn
here and do every conversion themselves.

The generator is counter-based (Philox), keyed by (base seed + config index,
CRC32 of the tensor's name), so a tensor's values depend only on its name,
shape and config - never on the order in which tensors are drawn.

Workload shapes stand in for the models the paper trains (Transformer base/big
and a GNMT-style LSTM stack, Section 5.1 and the configuration listing of
Section 2) on sub-word translation data with a ~32K vocabulary; sentence-length
variation, padding masks, dropout and label smoothing are left out on purpose.
"""
from __future__ import annotations

import math
import zlib
from dataclasses import dataclass, field, replace
from typing import Dict, List

import numpy as np

SEED_BASE = 0x180510387


def stream(config_index: int, name: str) -> np.random.Generator:
    key = np.array([(SEED_BASE + config_index) & 0xFFFFFFFFFFFFFFFF,
                    zlib.crc32(name.encode())], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def normal(config_index: int, name: str, shape, std: float = 1.0) -> np.ndarray:
    g = stream(config_index, name)
    return (g.standard_normal(size=shape, dtype=np.float64) * std).astype(np.float32)


def uniform(config_index: int, name: str, shape, a: float) -> np.ndarray:
    g = stream(config_index, name)
    return g.uniform(-a, a, size=shape).astype(np.float32)


def xavier_uniform(config_index: int, name: str, fan_out: int, fan_in: int,
                   shape=None) -> np.ndarray:
    a = math.sqrt(6.0 / (fan_in + fan_out))
    return uniform(config_index, name, shape or (fan_out, fan_in), a)


def zeros(shape) -> np.ndarray:
    return np.zeros(shape, dtype=np.float32)


def ones(shape) -> np.ndarray:
    return np.ones(shape, dtype=np.float32)


# --------------------------------------------------------------------------
# Workload descriptions
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class ScaleCfg:
    mode: str = "backoff"          # "static" | "backoff"
    init_scale: float = 2.0 ** 15
    growth_interval: int = 10
    min_scale: float = 1.0
    max_scale: float = 2.0 ** 24


@dataclass(frozen=True)
class OptCfg:
    kind: str = "adam"             # "sgd" | "adam"
    lr: float = 1e-4
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.0


@dataclass(frozen=True)
class MLPWorkload:
    """Config 1: two linear layers with a ReLU between, MSE loss, SGD."""
    index: int = 1
    rows: int = 64
    d_in: int = 256
    d_hidden: int = 1024
    d_out: int = 256
    steps: int = 20
    inject_step: int = 7           # 0-based; +inf written into w2's gradient
    opt: OptCfg = OptCfg(kind="sgd", lr=1e-2)
    scale: ScaleCfg = ScaleCfg(init_scale=2.0 ** 10, growth_interval=5)

    @property
    def tokens(self):
        return self.rows

    def masters(self) -> Dict[str, np.ndarray]:
        i = self.index
        return {
            "w1": normal(i, "w1", (self.d_hidden, self.d_in), 0.02),
            "b1": zeros((self.d_hidden,)),
            "w2": normal(i, "w2", (self.d_out, self.d_hidden), 0.02),
            "b2": zeros((self.d_out,)),
        }

    def batch(self) -> Dict[str, np.ndarray]:
        i = self.index
        return {"x": normal(i, "x", (self.rows, self.d_in)),
                "target": normal(i, "target", (self.rows, self.d_out))}


@dataclass(frozen=True)
class TransformerWorkload:
    """Configs 2 and 3: a stack of post-LayerNorm encoder layers, MSE loss, Adam."""
    index: int = 2
    n_layers: int = 1
    d_model: int = 512
    n_heads: int = 8
    d_ff: int = 2048
    seq_len: int = 64
    n_seq: int = 64
    steps: int = 50
    opt: OptCfg = OptCfg(kind="adam", lr=1e-4)
    scale: ScaleCfg = ScaleCfg(init_scale=2.0 ** 15, growth_interval=10)

    @property
    def tokens(self):
        return self.seq_len * self.n_seq

    @property
    def d_head(self):
        return self.d_model // self.n_heads

    def layer_masters(self, layer: int) -> Dict[str, np.ndarray]:
        i, d, f = self.index, self.d_model, self.d_ff
        p = f"l{layer}."
        # q, k, v projections are drawn as three d x d Xavier matrices and
        # stacked: rows [0,d) = q, [d,2d) = k, [2d,3d) = v.
        wqkv = np.concatenate([xavier_uniform(i, p + n, d, d) for n in ("wq", "wk", "wv")], axis=0)
        return {
            "wqkv": wqkv, "bqkv": zeros((3 * d,)),
            "wo": xavier_uniform(i, p + "wo", d, d), "bo": zeros((d,)),
            "ln1_g": ones((d,)), "ln1_b": zeros((d,)),
            "w1": xavier_uniform(i, p + "w1", f, d), "b1": zeros((f,)),
            "w2": xavier_uniform(i, p + "w2", d, f), "b2": zeros((d,)),
            "ln2_g": ones((d,)), "ln2_b": zeros((d,)),
        }

    def masters(self) -> List[Dict[str, np.ndarray]]:
        return [self.layer_masters(l) for l in range(self.n_layers)]

    def batch(self) -> Dict[str, np.ndarray]:
        i = self.index
        return {"x": normal(i, "x", (self.tokens, self.d_model)),
                "target": normal(i, "target", (self.tokens, self.d_model))}

    def n_params(self) -> int:
        d, f = self.d_model, self.d_ff
        return self.n_layers * (4 * d * d + 2 * d * f + 3 * d + d + f + d + 4 * d)

    def gemm_flops_per_step(self) -> float:
        """2*M*N*K over every contraction of forward + backward (dx and dw)."""
        t, d, f = self.tokens, self.d_model, self.d_ff
        proj = 4 * 2.0 * t * d * d
        ffn = 2 * 2.0 * t * d * f
        attn = 2 * 2.0 * t * self.seq_len * d
        return 3.0 * self.n_layers * (proj + ffn + attn)


@dataclass(frozen=True)
class XentWorkload:
    """Config 4: output projection to the vocabulary + softmax cross-entropy."""
    index: int = 4
    tokens: int = 8192
    d_model: int = 1024
    vocab: int = 32768
    steps: int = 8
    blowup_step: int = 3           # 0-based; row 0 of the hidden input x 1e4
    blowup_factor: float = 1e4
    opt: OptCfg = OptCfg(kind="adam", lr=1e-4)
    scale: ScaleCfg = ScaleCfg(init_scale=2.0 ** 15, growth_interval=4)

    def masters(self) -> Dict[str, np.ndarray]:
        return {"w": xavier_uniform(self.index, "w_vocab", self.vocab, self.d_model),
                "b": zeros((self.vocab,))}

    def batch(self) -> Dict[str, np.ndarray]:
        g = stream(self.index, "targets")
        return {"h": normal(self.index, "h", (self.tokens, self.d_model)),
                "targets": g.integers(0, self.vocab, size=(self.tokens,), dtype=np.int64).astype(np.int32)}


@dataclass(frozen=True)
class LSTMWorkload:
    """Config 5: stacked LSTM, gate contraction [4H x (I+H)] per time step, MSE on the top layer."""
    index: int = 5
    n_layers: int = 4
    hidden: int = 1024
    d_in: int = 1024
    batch_size: int = 32
    seq_len: int = 50
    steps: int = 20
    opt: OptCfg = OptCfg(kind="adam", lr=1e-4)
    scale: ScaleCfg = ScaleCfg(init_scale=2.0 ** 15, growth_interval=10)

    @property
    def tokens(self):
        return self.batch_size * self.seq_len

    def masters(self) -> List[Dict[str, np.ndarray]]:
        out = []
        for l in range(self.n_layers):
            i_dim = self.d_in if l == 0 else self.hidden
            out.append({"w": uniform(self.index, f"l{l}.w", (4 * self.hidden, i_dim + self.hidden), 0.1),
                        "b": zeros((4 * self.hidden,))})
        return out

    def batch(self) -> Dict[str, np.ndarray]:
        i = self.index
        return {"x": normal(i, "x", (self.seq_len, self.batch_size, self.d_in)),
                "target": normal(i, "target", (self.seq_len, self.batch_size, self.hidden))}


# The five configurations at full size ...
C1 = MLPWorkload()
C2 = TransformerWorkload(index=2)
C3 = TransformerWorkload(index=3, n_layers=6, d_model=1024, n_heads=16, d_ff=4096,
                         seq_len=128, n_seq=64, steps=3,
                         scale=ScaleCfg(init_scale=2.0 ** 15, growth_interval=100))
C4 = XentWorkload()
C5 = LSTMWorkload()

# ... and reduced versions of the same structure that a CPU finishes in
# seconds while still spanning several GEMM tiles and ragged tails.
C2_SMALL = replace(C2, d_model=192, n_heads=3, d_ff=328, seq_len=40, n_seq=5, steps=12,
                   scale=ScaleCfg(init_scale=2.0 ** 15, growth_interval=4))
C3_SMALL = replace(C3, n_layers=2, d_model=256, n_heads=4, d_ff=512, seq_len=48, n_seq=6, steps=3)
C4_SMALL = replace(C4, tokens=520, d_model=256, vocab=3000)
C5_SMALL = replace(C5, n_layers=2, hidden=128, d_in=96, batch_size=8, seq_len=6, steps=12,
                   scale=ScaleCfg(init_scale=2.0 ** 15, growth_interval=4))
