"""Training iterations of the five workloads as sequences of C-ABI calls.

Host control flow only: buffers are torch CUDA tensors used as raw device memory, and every
arithmetic step is a kernel of libmp.so.  The order follows the paper's statement of mixed-precision
training (Sections 3.1, 3.2): forward and loss-scaled backward on the fp16 copies, then one
mp_unscale_check_update over all parameters (inspect, then update masters or skip), then
mp_loss_scale_update.  Nothing here reads device memory, so a whole `step()` can be captured in a
HIP graph (`torch.cuda.graph`) and replayed.
"""
from __future__ import annotations

import math
from typing import Callable, Dict, List, Optional

import numpy as np
import torch

from . import _lib as ML
from . import binding as B

LN_EPS = 1e-5


def _round_up(n: int, k: int) -> int:
    return (n + k - 1) // k * k


class ParamStore:
    """fp32 masters, fp16 copies, fp16 gradients and Adam moments of a model, each kind in one
    contiguous device arena (every tensor starts on a 16-element boundary, gaps stay zero)."""

    def __init__(self, masters: Dict[str, np.ndarray], adam: bool):
        self.names = list(masters)
        self.shapes = {k: tuple(v.shape) for k, v in masters.items()}
        self.offsets, off = {}, 0
        for k, v in masters.items():
            self.offsets[k] = off
            off += _round_up(int(v.size), 16)
        self.total = off
        dev = "cuda"
        self.w32_arena = torch.zeros(off, dtype=torch.float32, device=dev)
        self.w16_arena = torch.zeros(off, dtype=torch.float16, device=dev)
        self.g16_arena = torch.zeros(off, dtype=torch.float16, device=dev)
        self.m_arena = torch.zeros(off, dtype=torch.float32, device=dev) if adam else None
        self.v_arena = torch.zeros(off, dtype=torch.float32, device=dev) if adam else None
        host = np.zeros(off, dtype=np.float32)
        for k, v in masters.items():
            host[self.offsets[k]:self.offsets[k] + v.size] = np.asarray(v, dtype=np.float32).reshape(-1)
        self.w32_arena.copy_(torch.from_numpy(host))
        B.mp_cast_f32_to_f16(off, self.w32_arena, self.w16_arena)     # fp16 copies = RNE16(masters)
        self.w32 = {k: self._view(self.w32_arena, k) for k in self.names}
        self.w16 = {k: self._view(self.w16_arena, k) for k in self.names}
        self.g16 = {k: self._view(self.g16_arena, k) for k in self.names}
        self.m = {k: self._view(self.m_arena, k) for k in self.names} if adam else {}
        self.v = {k: self._view(self.v_arena, k) for k in self.names} if adam else {}
        self.n_params = sum(int(np.prod(s)) for s in self.shapes.values())
        entries = [dict(g16=self.g16[k], w32=self.w32[k], w16=self.w16[k], m=self.m.get(k), v=self.v.get(k))
                   for k in self.names]
        self.tensor_list = B.tensor_list(entries)
        self.n_tensors = len(entries)
        flat = [dict(g16=self.g16_arena, w32=self.w32_arena, w16=self.w16_arena, m=self.m_arena, v=self.v_arena)]
        self.flat_list = B.tensor_list(flat)

    def _view(self, arena, k):
        n = int(np.prod(self.shapes[k]))
        return arena[self.offsets[k]:self.offsets[k] + n].view(self.shapes[k])


class _StepBase:
    def __init__(self, masters: Dict[str, np.ndarray], opt, scale_cfg, prechecked: bool = False, flat_update: bool = False):
        self.P = ParamStore(masters, adam=(opt.kind == "adam"))
        self.cfg = B.opt_cfg(opt.kind, opt.lr, opt.beta1, opt.beta2, opt.eps, opt.weight_decay)
        self.st = B.scale_state_alloc()
        mode = ML.MP_SCALE_BACKOFF if scale_cfg.mode == "backoff" else ML.MP_SCALE_STATIC
        B.mp_scale_state_init(self.st, mode, scale_cfg.init_scale, scale_cfg.growth_interval, scale_cfg.min_scale,
                              scale_cfg.max_scale)
        self.loss = torch.zeros(1, dtype=torch.float32, device="cuda")
        self.prechecked = prechecked
        self.flat_update = flat_update
        self.ws: Optional[torch.Tensor] = None
        # tests may set trace(name, layer, tensor): called right after the kernel that wrote `tensor`
        self.trace: Optional[Callable] = None
        # every gradient producer also reports non-finite outputs into the state itself, which is what
        # `prechecked` relies on to drop the separate inspection pass
        self.st_grad = self.st

    def _alloc_ws(self, nbytes: int):
        self.ws = torch.empty(_round_up(max(nbytes, 1024), 256) // 4, dtype=torch.float32, device="cuda")

    def optimizer(self):
        flags = ML.MP_UPDATE_PRECHECKED if self.prechecked else ML.MP_UPDATE_DEFAULT
        if self.flat_update:
            B.mp_unscale_check_update(self.P.flat_list, 1, self.cfg, self.st, flags)
        else:
            B.mp_unscale_check_update(self.P.tensor_list, self.P.n_tensors, self.cfg, self.st, flags)
        B.mp_loss_scale_update(self.st)

    def step(self, inject: Optional[Callable] = None):
        self.forward_backward()
        if inject is not None:
            inject(self.P.g16)
        self.optimizer()

    def state(self) -> B.ScaleState:
        return B.scale_state_read(self.st)

    def _t(self, name, layer, tensor):
        if self.trace is not None:
            self.trace(name, layer, tensor)


def _h16(x: np.ndarray) -> torch.Tensor:
    """Upload fp32 host data and round it to fp16 on the device (RNE, the library's cast)."""
    src = torch.from_numpy(np.ascontiguousarray(np.asarray(x, dtype=np.float32))).cuda()
    dst = torch.empty(src.shape, dtype=torch.float16, device="cuda")
    B.mp_cast_f32_to_f16(src.numel(), src, dst)
    return dst


# ====================================================================================== config 1
class MLPStep(_StepBase):
    """x -> relu(W1 x + b1) -> W2 h + b2, MSE loss (config 1)."""

    def __init__(self, wl, masters=None, **kw):
        super().__init__(masters or wl.masters(), wl.opt, wl.scale, **kw)
        self.wl = wl
        R, di, dh, do = wl.rows, wl.d_in, wl.d_hidden, wl.d_out
        e16 = lambda *s: torch.empty(s, dtype=torch.float16, device="cuda")
        self.x, self.target = e16(R, di), e16(R, do)
        self.h, self.y, self.dy, self.dpre, self.dx = e16(R, dh), e16(R, do), e16(R, do), e16(R, dh), e16(R, di)
        self.d1 = B.gemm_desc(R, dh, di, epilogue=ML.MP_EPI_BIAS_RELU)
        self.d2 = B.gemm_desc(R, do, dh, epilogue=ML.MP_EPI_BIAS)
        self._alloc_ws(max(B.mp_gemm_bwd_dw_workspace_bytes(self.d1, True), B.mp_gemm_bwd_dw_workspace_bytes(self.d2, True),
                           B.mp_loss_workspace_bytes(R, do)))

    def set_batch(self, batch):
        self.x.copy_(_h16(batch["x"]))
        self.target.copy_(_h16(batch["target"]))

    def forward_backward(self):
        w, g, st = self.P.w16, self.P.g16, self.st_grad
        R, do = self.wl.rows, self.wl.d_out
        B.mp_gemm_fwd(self.d1, self.x, w["w1"], w["b1"], None, self.h)
        B.mp_gemm_fwd(self.d2, self.h, w["w2"], w["b2"], None, self.y)
        B.mp_mse_scaled(R, do, self.y, self.target, do, self.st, self.loss, self.dy, self.ws)
        B.mp_gemm_bwd_dw(self.d2, self.dy, self.h, g["w2"], g["b2"], st, self.ws)
        B.mp_gemm_bwd_dx(self.d2, self.dy, w["w2"], self.dpre, relu_src=self.h, ld_aux=self.wl.d_hidden)
        B.mp_gemm_bwd_dw(self.d1, self.dpre, self.x, g["w1"], g["b1"], st, self.ws)
        B.mp_gemm_bwd_dx(self.d1, self.dpre, w["w1"], self.dx)


# ====================================================================================== configs 2, 3
class TransformerStep(_StepBase):
    """Stack of post-LayerNorm encoder layers with an MSE loss on the last output (configs 2, 3)."""

    def __init__(self, wl, masters=None, two_streams=False, fused_attention=True, grouped_dw=True, **kw):
        if masters is None:
            masters = {f"l{i}.{k}": v for i, lay in enumerate(wl.masters()) for k, v in lay.items()}
        super().__init__(masters, wl.opt, wl.scale, **kw)
        self.wl = wl
        self.two_streams = two_streams
        dk_ = wl.d_model // wl.n_heads
        # the fused attention kernels cover head size 64 and sequences up to 128 (multiple of 8); anything else
        # runs the unfused chain of batched products and softmax kernels
        self.fused_attention = fused_attention and dk_ == 64 and wl.seq_len <= 128 and wl.seq_len % 8 == 0
        self.alpha = 1.0 / math.sqrt(dk_)
        # one launch for the four weight-gradient products of a layer (each alone has too few tiles for the chip);
        # needs weight shapes in multiples of 128 and a token count in multiples of 64
        self.grouped_dw = (grouped_dw and wl.d_model % 128 == 0 and wl.d_ff % 128 == 0
                           and wl.tokens % 64 == 0)
        self._groups = {}
        self.side_stream = torch.cuda.Stream() if two_streams else None
        T, d, f, h, S, NB = wl.tokens, wl.d_model, wl.d_ff, wl.n_heads, wl.seq_len, wl.n_seq
        dk = d // h
        e16 = lambda *s: torch.empty(s, dtype=torch.float16, device="cuda")
        e32 = lambda *s: torch.empty(s, dtype=torch.float32, device="cuda")
        self.x0, self.target = e16(T, d), e16(T, d)
        self.act: List[dict] = []
        for _ in range(wl.n_layers):
            self.act.append(dict(qkv=e16(T, 3 * d), p=e16(NB, h, S, S), ctx=e16(T, d), a=e16(T, d), y1=e16(T, d),
                                 f=e16(T, f), g=e16(T, d), y2=e16(T, d), mean1=e32(T), rstd1=e32(T), mean2=e32(T),
                                 rstd2=e32(T)))
        # backward temporaries, shared by all layers
        self.gbuf = [e16(T, d), e16(T, d)]
        self.tmp = [dict(dz2=e16(T, d), df=e16(T, f), dz1=e16(T, d), dqkv=e16(T, 3 * d)) for _ in range(2)]
        self.dy1, self.dctx, self.dp = e16(T, d), e16(T, d), e16(NB, h, S, S)
        G = B.gemm_desc
        self.d_qkv = G(T, 3 * d, d, epilogue=ML.MP_EPI_BIAS)
        self.d_o = G(T, d, d, epilogue=ML.MP_EPI_BIAS)
        self.d_f1 = G(T, f, d, epilogue=ML.MP_EPI_BIAS_RELU)
        self.d_f2 = G(T, d, f, epilogue=ML.MP_EPI_BIAS)
        alpha = 1.0 / math.sqrt(dk)
        # scores = alpha q k^T and ctx = p v, batched over (sequence, head) with strides into qkv
        self.d_s = G(S, S, dk, ldx=3 * d, ldw=3 * d, ldy=S, alpha=alpha, batch_outer=NB, batch_inner=h,
                     sx=(S * 3 * d, dk), sw=(S * 3 * d, dk), sy=(h * S * S, S * S))
        self.d_c = G(S, dk, S, ldx=S, ldw=3 * d, ldy=d, trans_w=1, batch_outer=NB, batch_inner=h,
                     sx=(h * S * S, S * S), sw=(S * 3 * d, dk), sy=(S * d, dk))
        need = [B.mp_gemm_bwd_dw_workspace_bytes(x, True) for x in (self.d_qkv, self.d_o, self.d_f1, self.d_f2)]
        need += [B.mp_gemm_bwd_dw_workspace_bytes(self.d_s, False), B.mp_gemm_bwd_dw_workspace_bytes(self.d_c, False),
                 B.mp_layernorm_bwd_workspace_bytes(T, d), B.mp_loss_workspace_bytes(T, d)]
        self._alloc_ws(max(need))
        self.ws_side = torch.empty_like(self.ws)

    def set_batch(self, batch):
        self.x0.copy_(_h16(batch["x"]))
        self.target.copy_(_h16(batch["target"]))

    def forward(self):
        wl, w = self.wl, self.P.w16
        T, d, h, S, NB = wl.tokens, wl.d_model, wl.n_heads, wl.seq_len, wl.n_seq
        x = self.x0
        for l, a in enumerate(self.act):
            p = f"l{l}."
            B.mp_gemm_fwd(self.d_qkv, x, w[p + "wqkv"], w[p + "bqkv"], None, a["qkv"])
            if self.fused_attention:
                B.mp_attention_fwd(NB, h, S, d // h, a["qkv"], 3 * d, self.alpha, a["p"], a["ctx"], d)
            else:
                B.mp_gemm_fwd(self.d_s, a["qkv"], a["qkv"][:, d:], None, None, a["p"])
                self._t("s", l, a["p"])
                B.mp_softmax_fwd(NB * h * S, S, a["p"], a["p"], S)
                B.mp_gemm_fwd(self.d_c, a["p"], a["qkv"][:, 2 * d:], None, None, a["ctx"])
            B.mp_gemm_fwd(self.d_o, a["ctx"], w[p + "wo"], w[p + "bo"], None, a["a"])
            B.mp_layernorm_fwd(T, d, x, a["a"], w[p + "ln1_g"], w[p + "ln1_b"], LN_EPS, a["y1"], a["mean1"], a["rstd1"])
            B.mp_gemm_fwd(self.d_f1, a["y1"], w[p + "w1"], w[p + "b1"], None, a["f"])
            B.mp_gemm_fwd(self.d_f2, a["f"], w[p + "w2"], w[p + "b2"], None, a["g"])
            B.mp_layernorm_fwd(T, d, a["y1"], a["g"], w[p + "ln2_g"], w[p + "ln2_b"], LN_EPS, a["y2"], a["mean2"], a["rstd2"])
            x = a["y2"]
        return x

    def backward(self):
        """Backward pass.  The weight-gradient products do not feed anything else in the backward pass, so
        they are enqueued on a second stream (forked and joined with events, which HIP-graph capture records
        as parallel branches): their prologues, epilogues and partial last rounds overlap the input-gradient
        chain on the main stream.  Temporaries read by the side stream are double-buffered by layer parity, and
        the main stream waits for the side work of two layers back before reusing them."""
        wl, w, g, st, ws = self.wl, self.P.w16, self.P.g16, self.st_grad, self.ws
        T, d, f, h, S, NB = wl.tokens, wl.d_model, wl.d_ff, wl.n_heads, wl.seq_len, wl.n_seq
        main = torch.cuda.current_stream()
        side = self.side_stream if self.two_streams else None
        done = {}

        def fork(fn):
            """Run fn (weight-gradient calls) on the side stream after everything enqueued so far on main."""
            if side is None:
                fn(ws)
                return
            ev = torch.cuda.Event()
            ev.record(main)
            side.wait_event(ev)
            with torch.cuda.stream(side):
                fn(self.ws_side)

        # the layer-output gradient ping-pongs between two [T, d] buffers; the loss wrote gbuf[0]
        for i, l in enumerate(range(wl.n_layers - 1, -1, -1)):
            dy2, dx = self.gbuf[i % 2], self.gbuf[(i + 1) % 2]
            a, p = self.act[l], f"l{l}."
            tb = self.tmp[i % 2]
            dz2, df, dz1, dqkv = tb["dz2"], tb["df"], tb["dz1"], tb["dqkv"]
            if side is not None and i >= 2:
                main.wait_event(done[i - 2])        # side stream finished reading this parity's temporaries
            x = self.x0 if l == 0 else self.act[l - 1]["y2"]
            # dz2 is the gradient of g = W2 f + b2 too, so its column sums are b2's gradient
            B.mp_layernorm_bwd(T, d, dy2, a["y1"], a["g"], w[p + "ln2_g"], a["mean2"], a["rstd2"], dz2,
                               g[p + "ln2_g"], g[p + "ln2_b"], st, ws, dz_colsum=g[p + "b2"])
            self._t("dy2", l, dy2)
            self._t("dz2", l, dz2)
            if not self.grouped_dw:
                fork(lambda wsx: B.mp_gemm_bwd_dw(self.d_f2, dz2, a["f"], g[p + "w2"], None, st, wsx))
            B.mp_gemm_bwd_dx(self.d_f2, dz2, w[p + "w2"], df, relu_src=a["f"], ld_aux=f)
            self._t("df", l, df)
            if not self.grouped_dw:
                fork(lambda wsx: B.mp_gemm_bwd_dw(self.d_f1, df, a["y1"], g[p + "w1"], g[p + "b1"], st, wsx))
            B.mp_gemm_bwd_dx(self.d_f1, df, w[p + "w1"], self.dy1, add=dz2, ld_aux=d)
            self._t("dy1", l, self.dy1)
            B.mp_layernorm_bwd(T, d, self.dy1, x, a["a"], w[p + "ln1_g"], a["mean1"], a["rstd1"], dz1,
                               g[p + "ln1_g"], g[p + "ln1_b"], st, ws, dz_colsum=g[p + "bo"])
            self._t("dz1", l, dz1)
            if not self.grouped_dw:
                fork(lambda wsx: B.mp_gemm_bwd_dw(self.d_o, dz1, a["ctx"], g[p + "wo"], None, st, wsx))
            B.mp_gemm_bwd_dx(self.d_o, dz1, w[p + "wo"], self.dctx)
            self._t("dctx", l, self.dctx)
            # attention: dP = dctx V^T, dV = P^T dctx, dS = softmax', dQ = alpha dS K, dK = alpha dS^T Q
            if self.fused_attention:
                B.mp_attention_bwd(NB, h, S, d // h, a["qkv"], 3 * d, self.alpha, a["p"], self.dctx, d, dqkv, 3 * d)
            else:
                B.mp_gemm_bwd_dx(self.d_c, self.dctx, a["qkv"][:, 2 * d:], self.dp)
                self._t("dp", l, self.dp)
                B.mp_gemm_bwd_dw(self.d_c, self.dctx, a["p"], dqkv[:, 2 * d:], None, None, ws)
                B.mp_softmax_bwd(NB * h * S, S, a["p"], self.dp, self.dp, S)
                self._t("ds", l, self.dp)
                B.mp_gemm_bwd_dx(self.d_s, self.dp, a["qkv"][:, d:], dqkv)
                B.mp_gemm_bwd_dw(self.d_s, self.dp, a["qkv"], dqkv[:, d:], None, None, ws)
            self._t("dqkv", l, dqkv)
            if not self.grouped_dw:
                fork(lambda wsx: B.mp_gemm_bwd_dw(self.d_qkv, dqkv, x, g[p + "wqkv"], g[p + "bqkv"], st, wsx))
            B.mp_gemm_bwd_dx(self.d_qkv, dqkv, w[p + "wqkv"], dx, add=dz1, ld_aux=d)
            self._t("dx", l, dx)
            if self.grouped_dw:
                # all four operand pairs of this layer are still in place (the temporaries alternate by layer); the
                # two bias gradients that no LayerNorm backward produced ride in the same launch, on CUs that the
                # product tiles (fewer than the chip has CUs) leave idle
                key = (l, i % 2)
                if key not in self._groups:
                    self._groups[key] = B.gemm_group([(self.d_f2, dz2, a["f"], g[p + "w2"]),
                                                      (self.d_f1, df, a["y1"], g[p + "w1"], g[p + "b1"]),
                                                      (self.d_qkv, dqkv, x, g[p + "wqkv"], g[p + "bqkv"]),
                                                      (self.d_o, dz1, a["ctx"], g[p + "wo"])])
                fork(lambda wsx: B.mp_gemm_bwd_dw_grouped(self._groups[key], st))
            if side is not None:
                done[i] = torch.cuda.Event()
                done[i].record(side)
        if side is not None:
            main.wait_stream(side)                   # every weight gradient is complete before the update
        self.dx_input = self.gbuf[wl.n_layers % 2]

    def forward_backward(self):
        wl = self.wl
        y = self.forward()
        B.mp_mse_scaled(wl.tokens, wl.d_model, y, self.target, wl.d_model, self.st, self.loss, self.gbuf[0], self.ws)
        self.backward()


# ====================================================================================== config 4
class XentStep(_StepBase):
    """Hidden states -> vocabulary logits -> softmax cross-entropy (config 4)."""

    def __init__(self, wl, masters=None, **kw):
        super().__init__(masters or wl.masters(), wl.opt, wl.scale, **kw)
        self.wl = wl
        T, d, V = wl.tokens, wl.d_model, wl.vocab
        self.h = torch.empty(T, d, dtype=torch.float16, device="cuda")
        self.targets = torch.empty(T, dtype=torch.int32, device="cuda")
        self.logits = torch.empty(T, V, dtype=torch.float16, device="cuda")   # overwritten by dlogits
        self.dh = torch.empty(T, d, dtype=torch.float16, device="cuda")
        self.desc = B.gemm_desc(T, V, d, epilogue=ML.MP_EPI_BIAS)
        self._alloc_ws(max(B.mp_gemm_bwd_dw_workspace_bytes(self.desc, False), B.mp_softmax_xent_db_workspace_bytes(T, V)))

    def set_batch(self, batch):
        self.h.copy_(_h16(batch["h"]))
        self.targets.copy_(torch.from_numpy(np.asarray(batch["targets"], dtype=np.int32)).cuda())

    def forward_backward(self):
        wl, w, g = self.wl, self.P.w16, self.P.g16
        T, V = wl.tokens, wl.vocab
        B.mp_gemm_fwd(self.desc, self.h, w["w"], w["b"], None, self.logits)
        # the bias gradient (column sums of dlogits) comes out of the pass that writes dlogits
        B.mp_softmax_xent_scaled_db(T, V, self.logits, V, self.targets, self.st, self.loss, self.logits, g["b"], self.ws)
        B.mp_gemm_bwd_dw(self.desc, self.logits, self.h, g["w"], None, self.st_grad, self.ws)
        B.mp_gemm_bwd_dx(self.desc, self.logits, w["w"], self.dh)


# ====================================================================================== config 5
class LSTMStep(_StepBase):
    """Stacked LSTM unrolled over time with an MSE loss on the top layer's outputs (config 5).

    Layer l keeps xh[l][t] = [input_t | h_{t-1}] as one row block.  Two launch plans give the same stored tensors:

    persistent (default where the shape allows): per layer ONE large product for the input half of all gate sums
      (fp32, x W_x^T over all T*B rows), then ONE recurrent kernel that runs all T steps with the recurrent weights
      on chip (mp_lstm_layer_fwd); backward likewise one recurrent kernel per layer (mp_lstm_layer_bwd) followed by
      the large input-gradient and weight-gradient products over all T*B rows.
    step by step: per time step one gate product with W[4H, I+H] (mp_gemm_fwd_ws) and one cell kernel; the cell
      kernel writes h_t both into xh[l][t+1] (recurrence) and into the next layer's xh[l+1][t] (or the output)."""

    def __init__(self, wl, masters=None, persistent=True, **kw):
        if masters is None:
            masters = {f"l{i}.{k}": v for i, lay in enumerate(wl.masters()) for k, v in lay.items()}
        super().__init__(masters, wl.opt, wl.scale, **kw)
        self.wl = wl
        T, Bt, H, NL = wl.seq_len, wl.batch_size, wl.hidden, wl.n_layers
        z16 = lambda *s: torch.zeros(s, dtype=torch.float16, device="cuda")
        z32 = lambda *s: torch.zeros(s, dtype=torch.float32, device="cuda")
        self.in_dims = [wl.d_in if l == 0 else H for l in range(NL)]
        self.persistent = (persistent and Bt <= 32 and H % 128 == 0 and H <= 1024 and all(i % 8 == 0 for i in self.in_dims)
                           and H // 16 <= torch.cuda.get_device_properties(0).multi_processor_count)
        self.xh = [z16(T, Bt, self.in_dims[l] + H) for l in range(NL)]      # h_0 = 0 stays in xh[l][0][:, I:]
        self.gates = [z16(T, Bt, 4 * H) for _ in range(NL)]
        self.c = [z32(T + 1, Bt, H) for _ in range(NL)]                      # c_0 = 0
        self.y = z16(T, Bt, H)
        self.target = z16(T, Bt, H)
        self.dy = z16(T, Bt, H)
        self.dxh = [z16(T, Bt, max(self.in_dims) + H) for _ in range(2)]
        self.dgates = z16(T, Bt, 4 * H)
        self.dc = z32(Bt, H)
        self.d_gate = [B.gemm_desc(Bt, 4 * H, self.in_dims[l] + H, epilogue=ML.MP_EPI_BIAS) for l in range(NL)]
        self.d_gate_all = [B.gemm_desc(T * Bt, 4 * H, self.in_dims[l] + H) for l in range(NL)]
        need = [B.mp_gemm_bwd_dw_workspace_bytes(x, True) for x in self.d_gate_all] + [B.mp_loss_workspace_bytes(T * Bt, H)]
        # the recurrent products have only `batch` rows: with a workspace they split their contraction over the chip
        need += [B.mp_gemm_split_workspace_bytes(x) for x in self.d_gate]
        self._alloc_ws(max(need))
        if self.persistent:
            self.gx = z32(T * Bt, 4 * H)                                     # input half of the gate sums, all steps
            self.dx = [z16(T * Bt, max(self.in_dims)) for _ in range(2)]     # input gradient of a layer, all steps
            self.rl_status = torch.zeros(1, dtype=torch.int32, device="cuda")
            self.rl_ws = torch.zeros(B.mp_lstm_layer_workspace_bytes() // 4, dtype=torch.int32, device="cuda")
            # x W_x^T and dgates W_x: the input columns [0, I) of W[4H, I+H], all T*B rows at once
            self.d_in_all = [B.gemm_desc(T * Bt, 4 * H, self.in_dims[l], ldx=self.in_dims[l] + H, ldw=self.in_dims[l] + H)
                             for l in range(NL)]
            self.d_dx_all = [B.gemm_desc(T * Bt, 4 * H, self.in_dims[l], ldx=self.in_dims[l], ldw=self.in_dims[l] + H)
                             for l in range(NL)]

    def set_batch(self, batch):
        x = _h16(batch["x"])
        self.xh[0][:, :, :self.in_dims[0]].copy_(x)
        self.target.copy_(_h16(batch["target"]))

    def forward_backward(self):
        if self.persistent:
            self._forward_backward_persistent()
        else:
            self._forward_backward_stepwise()

    def recurrent_kernels_ok(self) -> bool:
        """False if a step barrier of a persistent kernel ever ran out of time (synchronises; tests and logging)."""
        return (not self.persistent) or int(self.rl_status.item()) == 0

    def _forward_backward_persistent(self):
        wl, w, g = self.wl, self.P.w16, self.P.g16
        T, Bt, H, NL = wl.seq_len, wl.batch_size, wl.hidden, wl.n_layers
        for l in range(NL):
            I = self.in_dims[l]
            B.mp_gemm_fwd(self.d_in_all[l], self.xh[l], w[f"l{l}.w"], None, None, None, self.gx)
            up, ldup = (self.xh[l + 1], self.in_dims[l + 1] + H) if l + 1 < NL else (self.y, H)
            d = B.lstm_layer_desc(T, Bt, I, H, I + H, I + H, ldup)
            B.mp_lstm_layer_fwd(d, self.gx, w[f"l{l}.w"], w[f"l{l}.b"], self.gates[l], self.c[l], self.xh[l], up,
                                self.rl_status, self.rl_ws)
        B.mp_mse_scaled(T * Bt, H, self.y, self.target, H, self.st, self.loss, self.dy, self.ws)
        above, ld_above = self.dy, H
        for l in range(NL - 1, -1, -1):
            I = self.in_dims[l]
            d = B.lstm_layer_desc(T, Bt, I, H, I + H, I + H, ld_above)
            B.mp_lstm_layer_bwd(d, w[f"l{l}.w"], self.gates[l], self.c[l], above, self.dgates, self.rl_status, self.rl_ws)
            dx = self.dx[l % 2].view(-1)[:T * Bt * I].view(T * Bt, I)
            B.mp_gemm_bwd_dx(self.d_dx_all[l], self.dgates, w[f"l{l}.w"], dx)
            B.mp_gemm_bwd_dw(self.d_gate_all[l], self.dgates, self.xh[l], g[f"l{l}.w"], g[f"l{l}.b"], self.st_grad, self.ws)
            above, ld_above = dx, I
        self.dx_input = above

    def _forward_backward_stepwise(self):
        wl, w, g = self.wl, self.P.w16, self.P.g16
        T, Bt, H, NL = wl.seq_len, wl.batch_size, wl.hidden, wl.n_layers
        for l in range(NL):
            I = self.in_dims[l]
            ldxh = I + H
            for t in range(T):
                B.mp_gemm_fwd_ws(self.d_gate[l], self.xh[l][t], w[f"l{l}.w"], w[f"l{l}.b"], None, self.gates[l][t], ws=self.ws)
                if l + 1 < NL:
                    up, ldup = self.xh[l + 1][t], self.in_dims[l + 1] + H
                else:
                    up, ldup = self.y[t], H
                rec = self.xh[l][t + 1][:, I:] if t + 1 < T else None
                B.mp_lstm_cell_fwd(Bt, H, self.gates[l][t], 4 * H, self.c[l][t], self.c[l][t + 1], up, ldup, rec, ldxh)
        B.mp_mse_scaled(T * Bt, H, self.y, self.target, H, self.st, self.loss, self.dy, self.ws)
        above, ld_above = self.dy, H
        for l in range(NL - 1, -1, -1):
            I = self.in_dims[l]
            ldxh = I + H
            dxh = self.dxh[l % 2].view(-1)[:T * Bt * ldxh].view(T, Bt, ldxh)
            B.mp_fill_u32(Bt * H, 0, self.dc)
            for t in range(T - 1, -1, -1):
                rec = dxh[t + 1][:, I:] if t + 1 < T else None
                B.mp_lstm_cell_bwd(Bt, H, self.gates[l][t], 4 * H, self.c[l][t], self.c[l][t + 1], above[t], ld_above,
                                   rec, ldxh, self.dc, self.dgates[t])
                B.mp_gemm_bwd_dx_ws(self.d_gate[l], self.dgates[t], w[f"l{l}.w"], dxh[t], ws=self.ws)
            B.mp_gemm_bwd_dw(self.d_gate_all[l], self.dgates, self.xh[l], g[f"l{l}.w"], g[f"l{l}.b"], self.st_grad, self.ws)
            above, ld_above = dxh, ldxh
        self.dx_input = above


# ====================================================================================== command line
def _main(argv=None):
    """python -m paper_1805_10387_amd.steps <1..5> [--steps N] [--warmup W] [--graph]
    Runs one of the five synthetic workloads for N timed iterations and prints one JSON line (ms per iteration,
    tokens or rows per second, final loss and scale state).  Meant for profiling a workload under rocprofv3."""
    import argparse
    import json
    import sys
    import os
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import mp_inputs as I
    ap = argparse.ArgumentParser(prog="python -m paper_1805_10387_amd.steps")
    ap.add_argument("config", type=int, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--graph", action="store_true", help="replay the iteration as a HIP graph")
    a = ap.parse_args(argv)
    wl = {1: I.C1, 2: I.C2, 3: I.C3, 4: I.C4, 5: I.C5}[a.config]
    # config 3 in the configuration bench.py times; the others as their parity tests run them
    kw = dict(prechecked=True, flat_update=True) if a.config == 3 else {}
    step = {1: MLPStep, 2: TransformerStep, 3: TransformerStep, 4: XentStep, 5: LSTMStep}[a.config](wl, **kw)
    step.set_batch(wl.batch())
    for _ in range(max(a.warmup, 1)):
        step.step()
    torch.cuda.synchronize()
    run = step.step
    if a.graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step.step()
        run = graph.replay
        run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(a.steps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / a.steps
    units = getattr(wl, "tokens", None) or getattr(wl, "rows", None) or 0
    s = step.state()
    print(json.dumps({"config": a.config, "ms_per_step": ms, "units_per_step": units, "units_per_s": units / (ms * 1e-3),
                      "parameters": int(step.P.total), "launch": "HIP graph replay" if a.graph else "eager",
                      "loss": float(step.loss), "loss_scale": s.scale, "opt_steps": s.opt_step, "skipped": s.skipped_steps}))


if __name__ == "__main__":
    _main()
