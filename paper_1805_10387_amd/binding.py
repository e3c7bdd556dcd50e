"""Thin Python binding of the C ABI in include/mp.h: same names, argument marshalling only.

Tensors are torch CUDA tensors used purely as device memory (`data_ptr()`); all work is
enqueued on torch's current stream by the HIP kernels of libmp.so."""
from __future__ import annotations

import ctypes as C
from typing import Optional, Sequence

import torch

from . import _lib as L
from ._lib import GemmDesc, OptCfg, ScaleState, TensorDesc  # noqa: F401


class MPError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libmp error {code}: {msg}")
        self.code = code


def _check(rc: int):
    if rc != 0:
        raise MPError(rc, L.load().mp_last_error().decode(errors="replace"))


def _p(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def mp_version() -> int:
    return L.load().mp_version()


# ------------------------------------------------------------------ scale state
def scale_state_alloc(device="cuda") -> torch.Tensor:
    """Device memory for one mp_scale_state (as int32 words)."""
    return torch.empty(C.sizeof(ScaleState) // 4, dtype=torch.int32, device=device)


def scale_state_read(st: torch.Tensor) -> ScaleState:
    """Host copy of the device state (synchronises; logging/tests only)."""
    host = st.cpu().numpy().tobytes()
    return ScaleState.from_buffer_copy(host)


def mp_scale_state_init(st, mode: int, init_scale: float, growth_interval: int, min_scale: float = 1.0,
                        max_scale: float = 2.0 ** 24):
    _check(L.load().mp_scale_state_init(_p(st), mode, init_scale, growth_interval, min_scale, max_scale, _stream()))


def mp_loss_scale_update(st):
    _check(L.load().mp_loss_scale_update(_p(st), _stream()))


# ------------------------------------------------------------------ contractions
def gemm_desc(M, N, K, ldx=None, ldw=None, ldy=None, trans_w=0, alpha=1.0, epilogue=L.MP_EPI_NONE,
              batch_outer=1, batch_inner=1, sx=(0, 0), sw=(0, 0), sy=(0, 0)) -> GemmDesc:
    d = GemmDesc()
    d.M, d.N, d.K = M, N, K
    d.ldx = K if ldx is None else ldx
    d.ldw = (N if trans_w else K) if ldw is None else ldw
    d.ldy = N if ldy is None else ldy
    d.batch_outer, d.batch_inner = batch_outer, batch_inner
    d.sx_outer, d.sx_inner = sx
    d.sw_outer, d.sw_inner = sw
    d.sy_outer, d.sy_inner = sy
    d.alpha, d.epilogue, d.trans_w = alpha, epilogue, trans_w
    return d


def mp_gemm_bwd_dw_workspace_bytes(desc: GemmDesc, with_db: bool) -> int:
    return L.load().mp_gemm_bwd_dw_workspace_bytes(C.byref(desc), int(with_db))


def mp_gemm_fwd(desc: GemmDesc, X, W, bias=None, acc_in=None, Y=None, y_f32=None):
    _check(L.load().mp_gemm_fwd(C.byref(desc), _p(X), _p(W), _p(bias), _p(acc_in), _p(Y), _p(y_f32), _stream()))


def mp_gemm_bwd_dx(desc: GemmDesc, dY, W, dX, relu_src=None, add=None, ld_aux=0):
    _check(L.load().mp_gemm_bwd_dx(C.byref(desc), _p(dY), _p(W), _p(relu_src), _p(add), ld_aux, _p(dX), _stream()))


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def mp_gemm_split_workspace_bytes(desc: GemmDesc) -> int:
    return L.load().mp_gemm_split_workspace_bytes(C.byref(desc))


def mp_gemm_fwd_ws(desc: GemmDesc, X, W, bias=None, acc_in=None, Y=None, y_f32=None, ws=None):
    _check(L.load().mp_gemm_fwd_ws(C.byref(desc), _p(X), _p(W), _p(bias), _p(acc_in), _p(Y), _p(y_f32), _p(ws), _nbytes(ws),
                                   _stream()))


def mp_gemm_bwd_dx_ws(desc: GemmDesc, dY, W, dX, relu_src=None, add=None, ld_aux=0, ws=None):
    _check(L.load().mp_gemm_bwd_dx_ws(C.byref(desc), _p(dY), _p(W), _p(relu_src), _p(add), ld_aux, _p(dX), _p(ws), _nbytes(ws),
                                      _stream()))


def mp_gemm_bwd_dw(desc: GemmDesc, dY, X, dW, db=None, st=None, ws=None):
    _check(L.load().mp_gemm_bwd_dw(C.byref(desc), _p(dY), _p(X), _p(dW), _p(db), _p(st), _p(ws),
                                   0 if ws is None else ws.numel() * ws.element_size(), _stream()))


def gemm_group(items):
    """Host array for mp_gemm_bwd_dw_grouped from (desc, dY, X, dW[, db]) tuples; keeps the tensors alive."""
    arr = (L.GemmGroupItem * len(items))()
    for k, it in enumerate(items):
        desc, dY, X, dW = it[:4]
        C.memmove(C.byref(arr[k].desc), C.byref(desc), C.sizeof(GemmDesc))
        arr[k].dY, arr[k].X, arr[k].dW = _p(dY), _p(X), _p(dW)
        arr[k].db = _p(it[4]) if len(it) > 4 else None
    arr._keep = [t for it in items for t in it[1:]]
    return arr


def mp_gemm_bwd_dw_grouped(group, st=None):
    _check(L.load().mp_gemm_bwd_dw_grouped(group, len(group), _p(st), _stream()))


def mp_gemm_tuning_override(tile: int, splits: int = 1):
    _check(L.load().mp_gemm_tuning_override(tile, splits))


def mp_gemm_tuning_dtl(mode: int):
    _check(L.load().mp_gemm_tuning_dtl(mode))


def mp_colsum_workspace_bytes(rows: int, cols: int) -> int:
    return L.load().mp_colsum_workspace_bytes(rows, cols)


def mp_colsum(rows, cols, dY, ld, db, st=None, ws=None):
    _check(L.load().mp_colsum(rows, cols, _p(dY), ld, _p(db), _p(st), _p(ws),
                              0 if ws is None else ws.numel() * ws.element_size(), _stream()))


def mp_colsum_static_max_bytes() -> int:
    return L.load().mp_colsum_static_max_bytes()


def mp_colsum_static(rows, cols, dY, ld, db, st=None):
    _check(L.load().mp_colsum_static(rows, cols, _p(dY), ld, _p(db), _p(st), _stream()))


# ------------------------------------------------------------------ losses
def mp_loss_workspace_bytes(rows: int, cols: int) -> int:
    return L.load().mp_loss_workspace_bytes(rows, cols)


def mp_mse_scaled(rows, cols, y, target, ld, st, loss, dy, ws):
    _check(L.load().mp_mse_scaled(rows, cols, _p(y), _p(target), ld, _p(st), _p(loss), _p(dy), _p(ws),
                                  ws.numel() * ws.element_size(), _stream()))


def mp_softmax_xent_scaled(rows, vocab, logits, ld, targets, st, loss, dlogits, ws):
    _check(L.load().mp_softmax_xent_scaled(rows, vocab, _p(logits), ld, _p(targets), _p(st), _p(loss), _p(dlogits),
                                           _p(ws), ws.numel() * ws.element_size(), _stream()))


def mp_softmax_xent_db_workspace_bytes(rows: int, vocab: int) -> int:
    return int(L.load().mp_softmax_xent_db_workspace_bytes(rows, vocab))


def mp_softmax_xent_scaled_db(rows, vocab, logits, ld, targets, st, loss, dlogits, db, ws):
    _check(L.load().mp_softmax_xent_scaled_db(rows, vocab, _p(logits), ld, _p(targets), _p(st), _p(loss), _p(dlogits),
                                              _p(db), _p(ws), ws.numel() * ws.element_size(), _stream()))


# ------------------------------------------------------------------ bandwidth-bound pieces
def mp_layernorm_fwd(rows, d, x, a, gamma, beta, eps, y, mean, rstd):
    _check(L.load().mp_layernorm_fwd(rows, d, _p(x), _p(a), _p(gamma), _p(beta), eps, _p(y), _p(mean), _p(rstd), _stream()))


def mp_layernorm_bwd_workspace_bytes(rows: int, d: int) -> int:
    return L.load().mp_layernorm_bwd_workspace_bytes(rows, d)


def mp_layernorm_bwd(rows, d, dy, x, a, gamma, mean, rstd, dz, dgamma, dbeta, st, ws, dz_colsum=None):
    _check(L.load().mp_layernorm_bwd(rows, d, _p(dy), _p(x), _p(a), _p(gamma), _p(mean), _p(rstd), _p(dz), _p(dgamma),
                                     _p(dbeta), _p(dz_colsum), _p(st), _p(ws), ws.numel() * ws.element_size(), _stream()))


def mp_softmax_fwd(rows, cols, s, p, ld):
    _check(L.load().mp_softmax_fwd(rows, cols, _p(s), _p(p), ld, _stream()))


def mp_softmax_bwd(rows, cols, p, dp, ds, ld):
    _check(L.load().mp_softmax_bwd(rows, cols, _p(p), _p(dp), _p(ds), ld, _stream()))


def mp_attention_fwd(n_seq, n_heads, seq_len, d_head, qkv, ld_qkv, alpha, p, ctx, ld_ctx):
    _check(L.load().mp_attention_fwd(n_seq, n_heads, seq_len, d_head, _p(qkv), ld_qkv, alpha, _p(p), _p(ctx), ld_ctx, _stream()))


def mp_attention_bwd(n_seq, n_heads, seq_len, d_head, qkv, ld_qkv, alpha, p, dctx, ld_ctx, dqkv, ld_dqkv):
    _check(L.load().mp_attention_bwd(n_seq, n_heads, seq_len, d_head, _p(qkv), ld_qkv, alpha, _p(p), _p(dctx), ld_ctx,
                                     _p(dqkv), ld_dqkv, _stream()))


def mp_lstm_cell_fwd(B, H, gates, ldg, c_prev, c, h_out, ldh, h_out2=None, ldh2=0):
    _check(L.load().mp_lstm_cell_fwd(B, H, _p(gates), ldg, _p(c_prev), _p(c), _p(h_out), ldh, _p(h_out2), ldh2, _stream()))


def mp_lstm_cell_bwd(B, H, gates, ldg, c_prev, c, dh_a, ld_a, dh_b, ld_b, dc, dgates):
    _check(L.load().mp_lstm_cell_bwd(B, H, _p(gates), ldg, _p(c_prev), _p(c), _p(dh_a), ld_a, _p(dh_b), ld_b, _p(dc),
                                     _p(dgates), _stream()))


def lstm_layer_desc(T, B, I, H, ldw, ldxh, ld_up, wait_limit_us=0, debug_extra_participants=0) -> L.LstmLayerDesc:
    return L.LstmLayerDesc(T, B, I, H, ldw, ldxh, ld_up, wait_limit_us, debug_extra_participants, 0)


def mp_lstm_layer_workspace_bytes() -> int:
    return L.load().mp_lstm_layer_workspace_bytes()


def mp_lstm_layer_fwd(desc, gx, w, bias, gates, c, xh, h_up, status, ws):
    _check(L.load().mp_lstm_layer_fwd(C.byref(desc), _p(gx), _p(w), _p(bias), _p(gates), _p(c), _p(xh), _p(h_up), _p(status),
                                      _p(ws), ws.numel() * ws.element_size(), _stream()))


def mp_lstm_layer_bwd(desc, w, gates, c, dh_above, dgates, status, ws):
    _check(L.load().mp_lstm_layer_bwd(C.byref(desc), _p(w), _p(gates), _p(c), _p(dh_above), _p(dgates), _p(status), _p(ws),
                                      ws.numel() * ws.element_size(), _stream()))


def mp_cast_f32_to_f16(n, src, dst):
    _check(L.load().mp_cast_f32_to_f16(n, _p(src), _p(dst), _stream()))


def mp_fill_u32(n, value, dst):
    _check(L.load().mp_fill_u32(n, value, _p(dst), _stream()))


def mp_mfma_sustained_rate(operands, sink, workgroups: int, iters: int) -> float:
    """TFLOP/s the matrix cores sustain with the given operand values held in registers (blocks)."""
    out = C.c_double(0.0)
    _check(L.load().mp_mfma_sustained_rate(_p(operands), operands.numel(), _p(sink), sink.numel(), workgroups, iters,
                                           C.byref(out), _stream()))
    return out.value


# ------------------------------------------------------------------ optimizer wrapper
def opt_cfg(kind: str, lr: float, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0) -> OptCfg:
    c = OptCfg()
    c.kind = {"sgd": L.MP_OPT_SGD, "adam": L.MP_OPT_ADAM}[kind]
    c.lr, c.beta1, c.beta2, c.eps, c.weight_decay = lr, beta1, beta2, eps, weight_decay
    return c


def tensor_list(entries: Sequence[dict]):
    """Host array of mp_tensor_desc from dicts of torch tensors {g16, w32, w16, m, v}."""
    arr = (TensorDesc * len(entries))()
    for i, e in enumerate(entries):
        arr[i].g16, arr[i].w32, arr[i].w16 = _p(e["g16"]), _p(e["w32"]), _p(e["w16"])
        arr[i].m, arr[i].v = _p(e.get("m")), _p(e.get("v"))
        arr[i].n = e["w32"].numel()
    return arr


def mp_unscale_check_update(tensors, ntensors: int, cfg: OptCfg, st, flags: int = L.MP_UPDATE_DEFAULT):
    _check(L.load().mp_unscale_check_update(tensors, ntensors, C.byref(cfg), _p(st), flags, _stream()))
