"""End-to-end parity of whole training iterations (HIP library through its C ABI) against the CPU oracle.

Two protocols, both on the same seeded inputs:
  * teacher-forced: at every step the oracle recomputes loss and gradients from the weights the GPU holds,
    and re-applies the optimizer wrapper to the GPU's own pre-update state and gradients.  This checks each
    iteration to the benchmark spec's tolerances (gradients rel. Frobenius <= 1e-3, masters <= 1e-5, flags/scale
    state exact) without letting Adam's sign-like first steps amplify 1-ulp gradient differences.
  * free-running: oracle and GPU train independently; the overflow flags, skipped steps and the loss-scale
    sequence must agree exactly, losses closely.
"""
from dataclasses import replace

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_1805_10387_amd as mp
from paper_1805_10387_amd import steps as St
import mp_inputs as I
from oracle import MIXED, FP64
from oracle import layers as L
from oracle import models as Mo
from oracle import optimizer as O
from oracle.numerics import half_bits
from gpu_util import *

GRAD_TOL, MASTER_TOL = 1e-3, 1e-5


def _flat(wl):
    m = wl.masters()
    return Mo.flatten_layers(m) if isinstance(m, list) else m


def _snapshot(step):
    P = step.P
    return dict(w16={k: np32(P.w16[k]) for k in P.names}, w32={k: np32(P.w32[k]) for k in P.names},
                m={k: np32(P.m[k]) for k in P.names} if P.m else {}, v={k: np32(P.v[k]) for k in P.names} if P.v else {})


def _f64(d):
    return {k: (v if np.issubdtype(np.asarray(v).dtype, np.integer) else np.asarray(v, np.float64)) for k, v in d.items()}


def teacher_forced(step, wl, fwd_bwd, batch, n_steps, inject_at=None, inject_name=None, expect_found=(),
                   loss_tol=2e-4, batch_fn=None, grad_mode="direct", progress=None):
    """grad_mode "direct": whole-network gradients within GRAD_TOL of the oracle's (holds where the network
    has no discontinuity between the compared tensors and identical inputs).  "vs_fp64": for deep ReLU
    stacks a 1-ulp difference in a stored activation flips ReLU masks and moves whole-network gradients by
    ~1e-2 - exactly as far as the oracle itself sits from the fp64 definition - so the whole-network check
    is that the GPU is as close to the fp64 gradients as the oracle is; the 1e-3 bound is then enforced op
    by op on in-situ data (op_level_transformer)."""
    names = step.P.names
    worst = dict(grad=0.0, master=0.0)
    for k in range(n_steps):
        if batch_fn is not None:
            batch = batch_fn(k)
            step.set_batch(batch)
        ob = Mo.island_batch(MIXED, batch)
        before, s0 = _snapshot(step), step.state()
        step.forward_backward()
        if inject_at is not None and k == inject_at:
            step.P.g16[inject_name].view(-1)[0:1].fill_(float("inf"))
        g_gpu = {n: np32(step.P.g16[n]) for n in names}
        loss_ref, g_ref = fwd_bwd(MIXED, before["w16"], ob, float(s0.scale))
        if inject_at is not None and k == inject_at:
            g_ref[inject_name].reshape(-1)[0] = np.inf
        ref_bad = O.has_nonfinite(MIXED, list(g_ref.values()))
        assert ref_bad == (k in expect_found), f"step {k}: oracle overflow={ref_bad}"
        if np.isfinite(float(loss_ref)):
            assert abs(float(step.loss) - float(loss_ref)) <= loss_tol * abs(float(loss_ref)), (k, float(step.loss), float(loss_ref))
        else:
            assert not np.isfinite(float(step.loss))
        if not ref_bad and grad_mode == "direct":
            for n in names:
                e = rel_fro(g_gpu[n], g_ref[n])
                worst["grad"] = max(worst["grad"], e)
                assert e <= GRAD_TOL, f"step {k} grad {n}: rel Frobenius {e:.2e}"
        elif not ref_bad:
            _, g64 = fwd_bwd(FP64, _f64(before["w16"]), _f64(ob), float(s0.scale))
            for n in names:
                e_gpu, e_orc = rel_fro(g_gpu[n], g64[n]), rel_fro(g_ref[n], g64[n])
                worst["grad"] = max(worst["grad"], e_gpu)
                assert e_gpu <= 3.0 * e_orc + GRAD_TOL, f"step {k} grad {n}: GPU {e_gpu:.2e} vs oracle {e_orc:.2e} from fp64"
        else:
            assert O.has_nonfinite(MIXED, list(g_gpu.values()))
        # oracle's optimizer wrapper on the GPU's own state and gradients
        tensors = [dict(g16=g_gpu[n], w32=before["w32"][n].copy(), w16=before["w16"][n].copy(),
                        m=before["m"].get(n, np.zeros(1, np.float32)).copy(), v=before["v"].get(n, np.zeros(1, np.float32)).copy())
                   for n in names]
        ost = O.ScaleState(mode=wl.scale.mode, scale=float(s0.scale), growth_interval=s0.growth_interval,
                           min_scale=float(s0.min_scale), max_scale=float(s0.max_scale), good_steps=s0.good_steps,
                           opt_step=s0.opt_step, total_steps=s0.total_steps, skipped_steps=s0.skipped_steps)
        found = O.unscale_check_update(MIXED, tensors, wl.opt, ost)
        O.loss_scale_update(ost, found)
        step.optimizer()
        s1, after = step.state(), _snapshot(step)
        assert found == int(k in expect_found)
        assert (s1.scale, s1.good_steps, s1.opt_step, s1.total_steps, s1.skipped_steps, s1.found_inf) == \
               (ost.scale, ost.good_steps, ost.opt_step, ost.total_steps, ost.skipped_steps, 0), f"step {k} state"
        assert s1.hist_scale[k] == s0.scale and s1.hist_found_inf[k] == found
        for n, t in zip(names, tensors):
            if found:
                assert after["w32"][n].tobytes() == before["w32"][n].tobytes() and after["w16"][n].tobytes() == before["w16"][n].tobytes()
                continue
            e = rel_fro(after["w32"][n], t["w32"])
            worst["master"] = max(worst["master"], e)
            assert e <= MASTER_TOL, f"step {k} master {n}: {e:.2e}"
            assert np.array_equal(half_bits(after["w16"][n]), half_bits(MIXED.store(after["w32"][n]))), f"w16 != RNE16(w32) for {n}"
            if after["m"]:
                assert rel_fro(after["m"][n], t["m"]) <= MASTER_TOL and rel_fro(after["v"][n], t["v"]) <= MASTER_TOL
        if progress:
            print(f"{progress}: step {k} loss {float(step.loss):.5f} worst so far {worst}", flush=True)
    return worst


def free_running(step, wl, fwd_bwd, batch, n_steps, inject_at=None, inject_name=None, batch_fn=None, loss_tol=2e-3):
    tr = Mo.Trainer(MIXED, _flat(wl), wl.opt, wl.scale)
    losses = []
    for k in range(n_steps):
        if batch_fn is not None:
            batch = batch_fn(k)
            step.set_batch(batch)
        inj_o = inj_g = None
        if inject_at is not None and k == inject_at:
            def inj_o(grads):
                grads[inject_name].reshape(-1)[0] = np.inf

            def inj_g(g16):
                g16[inject_name].view(-1)[0:1].fill_(float("inf"))
        tr.step(fwd_bwd, Mo.island_batch(MIXED, batch), inj_o)
        step.step(inj_g)
        losses.append(float(step.loss))
    s = step.state()
    assert [s.hist_scale[i] for i in range(n_steps)] == [h[0] for h in tr.state.history]
    assert [s.hist_found_inf[i] for i in range(n_steps)] == [h[1] for h in tr.state.history]
    assert (s.scale, s.good_steps, s.opt_step, s.skipped_steps) == (tr.state.scale, tr.state.good_steps, tr.state.opt_step, tr.state.skipped_steps)
    assert np.allclose(losses, tr.losses, rtol=loss_tol, equal_nan=True), (losses, tr.losses)
    return tr, losses


def _graph_step(step):
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step.step()
    return g


# ------------------------------------------------------------------ config 1 (full size)
def test_config1_teacher_forced():
    wl = I.C1
    step = St.MLPStep(wl)
    batch = wl.batch()
    step.set_batch(batch)
    teacher_forced(step, wl, Mo.mlp_fwd_bwd, batch, wl.steps, inject_at=wl.inject_step, inject_name="w2",
                   expect_found={wl.inject_step})


def test_config1_free_running_sequence_and_masters():
    from test_oracle_optimizer import _golden
    wl = I.C1
    step = St.MLPStep(wl)
    batch = wl.batch()
    step.set_batch(batch)
    tr, losses = free_running(step, wl, Mo.mlp_fwd_bwd, batch, wl.steps, inject_at=wl.inject_step, inject_name="w2")
    g = _golden()["c1"]
    s = step.state()
    assert [s.hist_scale[i] for i in range(20)] == g["seq"] and (s.scale, s.good_steps, s.opt_step, s.skipped_steps) == (g["final"], g["good"], g["t"], g["skipped"])
    for n in ("w1", "w2"):                        # SGD: no sign-like amplification, masters stay within 1e-5
        assert rel_fro(np32(step.P.w32[n]), tr.w32[n]) <= MASTER_TOL, n
    for n in ("b1", "b2"):                        # zero-initialised: the master IS -lr * sum of gradients
        assert rel_fro(np32(step.P.w32[n]), tr.w32[n]) <= GRAD_TOL, n


def test_config1_static_scale_that_is_not_a_power_of_two():
    """Section 3.1 allows a constant loss scale of any value: S = 1000 for the whole run, the injected overflow
    skips its step and leaves S alone.  Unscaling by a non-power-of-two is not exact, so this also exercises the
    rounding of g / S on both sides."""
    wl = replace(I.C1, scale=I.ScaleCfg(mode="static", init_scale=1000.0))
    batch = wl.batch()
    step = St.MLPStep(wl)
    step.set_batch(batch)
    teacher_forced(step, wl, Mo.mlp_fwd_bwd, batch, 10, inject_at=wl.inject_step, inject_name="w2",
                   expect_found={wl.inject_step})
    step = St.MLPStep(wl)
    step.set_batch(batch)
    tr, _ = free_running(step, wl, Mo.mlp_fwd_bwd, batch, 12, inject_at=wl.inject_step, inject_name="w2")
    s = step.state()
    assert [s.hist_scale[i] for i in range(12)] == [1000.0] * 12
    assert (s.scale, s.opt_step, s.skipped_steps) == (1000.0, 11, 1)
    for n in ("w1", "w2"):
        assert rel_fro(np32(step.P.w32[n]), tr.w32[n]) <= MASTER_TOL, n


def test_config1_exponentially_decaying_learning_rate():
    """The learning rate is an argument of every optimizer call, so a schedule is host arithmetic: lr_k = lr_0 0.8^k
    on both sides, masters compared after 12 steps (SGD: no sign-like amplification)."""
    wl = I.C1
    batch = wl.batch()
    step = St.MLPStep(wl)
    step.set_batch(batch)
    w0 = _flat(wl)
    tr = Mo.Trainer(MIXED, w0, wl.opt, wl.scale)
    ob = Mo.island_batch(MIXED, batch)
    for k in range(12):
        lr = wl.opt.lr * 0.8 ** k
        tr.opt = replace(wl.opt, lr=lr)
        step.cfg.lr = lr
        tr.step(Mo.mlp_fwd_bwd, ob)
        step.step()
    s = step.state()
    assert (s.opt_step, s.skipped_steps, s.scale) == (tr.state.opt_step, tr.state.skipped_steps, tr.state.scale)
    for n in ("w1", "w2"):
        assert rel_fro(np32(step.P.w32[n]), tr.w32[n]) <= MASTER_TOL, n
        assert rel_fro(np32(step.P.w32[n]) - w0[n], tr.w32[n] - w0[n]) <= GRAD_TOL, n  # the movement itself
        assert np.array_equal(half_bits(np32(step.P.w16[n])), half_bits(MIXED.store(np32(step.P.w32[n]))))


# ------------------------------------------------------------------ configs 2, 3
def op_level_transformer(step, wl, batch, tol=GRAD_TOL, layers=None):
    """One forward/backward on the GPU with every stored tensor captured; each operation of the oracle is then
    evaluated on the GPU's own inputs of that operation and compared with the GPU's output of it."""
    tr = {}
    step.trace = lambda name, l, t: tr.__setitem__((name, l), np32(t))
    w = {k: np32(step.P.w16[k]) for k in step.P.names}
    scale = float(step.state().scale)
    step.forward_backward()
    step.trace = None
    g = {k: np32(step.P.g16[k]) for k in step.P.names}
    acts = [{k: np32(v) for k, v in a.items()} for a in step.act]
    NB, S, h, d = wl.n_seq, wl.seq_len, wl.n_heads, wl.d_model
    worst = [0.0]

    def check(got, ref, what):
        e = rel_fro(got, ref)
        worst[0] = max(worst[0], e)
        assert e <= tol, f"{what}: rel Frobenius {e:.2e}"

    def heads(qkv):
        return (L._heads(qkv[:, :d], NB, S, h), L._heads(qkv[:, d:2 * d], NB, S, h), L._heads(qkv[:, 2 * d:], NB, S, h))

    x = np32(step.x0)
    xs = []
    alpha = np.float32(1.0 / np.sqrt(d // h))
    layers = tuple(range(wl.n_layers)) if layers is None else tuple(layers)
    for l in range(wl.n_layers):
        a, p = acts[l], f"l{l}."
        xs.append(x)
        if l not in layers:
            x = a["y2"]
            continue
        check(a["qkv"], L.linear_fwd(MIXED, x, w[p + "wqkv"], w[p + "bqkv"]), f"{l} qkv")
        q, k, v = heads(a["qkv"])
        if ("s", l) in tr:
            check(tr[("s", l)], MIXED.store(alpha * (q @ k.transpose(0, 1, 3, 2))), f"{l} scores")
            check(a["p"], MIXED.store(L.softmax_rows(MIXED, tr[("s", l)])), f"{l} softmax")
        else:                                       # fused attention: scores never reach memory
            check(a["p"], MIXED.store(L.softmax_rows(MIXED, MIXED.store(alpha * (q @ k.transpose(0, 1, 3, 2))))), f"{l} softmax(scores)")
        check(a["ctx"], L._unheads(MIXED.store(a["p"] @ v)), f"{l} ctx")
        check(a["a"], L.linear_fwd(MIXED, a["ctx"], w[p + "wo"], w[p + "bo"]), f"{l} attn out")
        y1, c1 = L.layernorm_fwd(MIXED, x, a["a"], w[p + "ln1_g"], w[p + "ln1_b"])
        check(a["y1"], y1, f"{l} ln1")
        check(a["rstd1"], c1[1][:, 0], f"{l} rstd1")
        check(a["f"], L.linear_fwd(MIXED, a["y1"], w[p + "w1"], w[p + "b1"], relu=True), f"{l} ffn1")
        check(a["g"], L.linear_fwd(MIXED, a["f"], w[p + "w2"], w[p + "b2"]), f"{l} ffn2")
        y2, _ = L.layernorm_fwd(MIXED, a["y1"], a["g"], w[p + "ln2_g"], w[p + "ln2_b"])
        check(a["y2"], y2, f"{l} ln2")
        x = a["y2"]
    loss_ref, dy_ref = L.mse_scaled(MIXED, x, np32(step.target), scale)
    assert abs(float(step.loss) - float(loss_ref)) <= 1e-5 * float(loss_ref)
    check(tr[("dy2", wl.n_layers - 1)], dy_ref, "seed gradient")
    for l in range(wl.n_layers - 1, -1, -1):
        if l not in layers:
            continue
        a, p, x = acts[l], f"l{l}.", xs[l]
        _, c2 = L.layernorm_fwd(MIXED, a["y1"], a["g"], w[p + "ln2_g"], w[p + "ln2_b"])
        dz2, dg, db = L.layernorm_bwd(MIXED, tr[("dy2", l)], c2, w[p + "ln2_g"])
        check(tr[("dz2", l)], dz2, f"{l} dz2"); check(g[p + "ln2_g"], dg, f"{l} dln2_g"); check(g[p + "ln2_b"], db, f"{l} dln2_b")
        df, dw, db = L.linear_bwd(MIXED, tr[("dz2", l)], a["f"], w[p + "w2"])
        check(g[p + "w2"], dw, f"{l} dw2"); check(g[p + "b2"], db, f"{l} db2")
        check(tr[("df", l)], L.relu_mask(MIXED, df, a["f"]), f"{l} df")
        dy1, dw, db = L.linear_bwd(MIXED, tr[("df", l)], a["y1"], w[p + "w1"])
        check(g[p + "w1"], dw, f"{l} dw1"); check(g[p + "b1"], db, f"{l} db1")
        check(tr[("dy1", l)], L.add_store(MIXED, dy1, tr[("dz2", l)]), f"{l} dy1")
        _, c1 = L.layernorm_fwd(MIXED, x, a["a"], w[p + "ln1_g"], w[p + "ln1_b"])
        dz1, dg, db = L.layernorm_bwd(MIXED, tr[("dy1", l)], c1, w[p + "ln1_g"])
        check(tr[("dz1", l)], dz1, f"{l} dz1"); check(g[p + "ln1_g"], dg, f"{l} dln1_g"); check(g[p + "ln1_b"], db, f"{l} dln1_b")
        dctx, dw, db = L.linear_bwd(MIXED, tr[("dz1", l)], a["ctx"], w[p + "wo"])
        check(g[p + "wo"], dw, f"{l} dwo"); check(g[p + "bo"], db, f"{l} dbo"); check(tr[("dctx", l)], dctx, f"{l} dctx")
        q, k, v = heads(a["qkv"])
        dctx_h = L._heads(tr[("dctx", l)], NB, S, h)
        pg = a["p"]
        if ("dp", l) in tr:
            check(tr[("dp", l)], MIXED.store(dctx_h @ v.transpose(0, 1, 3, 2)), f"{l} dp")
            dpg = tr[("dp", l)]
            check(tr[("ds", l)], MIXED.store(pg * (dpg - (dpg * pg).sum(-1, keepdims=True, dtype=np.float32))), f"{l} ds")
            dsg = tr[("ds", l)]
        else:                                       # fused attention: dP and dS stay on chip; follow the oracle's own
            dpg = MIXED.store(dctx_h @ v.transpose(0, 1, 3, 2))
            dsg = MIXED.store(pg * (dpg - (dpg * pg).sum(-1, keepdims=True, dtype=np.float32)))
        dqkv = np.concatenate([L._unheads(MIXED.store(alpha * (dsg @ k))),
                               L._unheads(MIXED.store(alpha * (dsg.transpose(0, 1, 3, 2) @ q))),
                               L._unheads(MIXED.store(pg.transpose(0, 1, 3, 2) @ dctx_h))], axis=1)
        check(tr[("dqkv", l)], dqkv, f"{l} dqkv")
        dxa, dw, db = L.linear_bwd(MIXED, tr[("dqkv", l)], x, w[p + "wqkv"])
        check(g[p + "wqkv"], dw, f"{l} dwqkv"); check(g[p + "bqkv"], db, f"{l} dbqkv")
        check(tr[("dx", l)], L.add_store(MIXED, dxa, tr[("dz1", l)]), f"{l} dx")
    return worst[0]


def _transformer(wl, n_tf, n_free, **kw):
    f = Mo.make_transformer_fwd_bwd(wl.n_layers, wl.n_seq, wl.seq_len, wl.n_heads)
    batch = wl.batch()
    step = St.TransformerStep(wl, **kw)
    step.set_batch(batch)
    op_level_transformer(step, wl, batch)
    worst = teacher_forced(step, wl, f, batch, n_tf, grad_mode="vs_fp64")
    if n_free:
        step2 = St.TransformerStep(wl, **kw)
        step2.set_batch(batch)
        free_running(step2, wl, f, batch, n_free)
    return worst


def test_config2_reduced_size():
    _transformer(I.C2_SMALL, 6, I.C2_SMALL.steps)


def test_config3_reduced_size_two_layers():
    _transformer(I.C3_SMALL, 3, 3)


def test_unfused_attention_path_reduced_size():
    """The chain of batched products and softmax kernels (used where the fused kernel does not apply)."""
    wl = I.C3_SMALL
    batch = wl.batch()
    step = St.TransformerStep(wl, fused_attention=False)
    step.set_batch(batch)
    assert not step.fused_attention
    op_level_transformer(step, wl, batch)


def test_config3_reduced_prechecked_flat_update_matches_default():
    """The bench launch configuration (producer-side inspection, one flat descriptor) gives the same bits."""
    wl, batch = I.C3_SMALL, I.C3_SMALL.batch()
    a, b = St.TransformerStep(wl), St.TransformerStep(wl, prechecked=True, flat_update=True)
    for s in (a, b):
        s.set_batch(batch)
        for _ in range(3):
            s.step()
    assert torch.equal(a.P.w32_arena, b.P.w32_arena) and torch.equal(a.P.w16_arena, b.P.w16_arena)
    assert float(a.loss) == float(b.loss)


def _assert_clean_steps_have_margin(step, lo=0.55, hi=0.8):
    """The largest finite |gradient| of a clean step, as a fraction of the fp16 maximum.  Inside (lo, hi) the skip
    decisions of a run are not a matter of summation order: the same step one scale doubling up overflows by more than
    10 %, and stays clean by more than 20 %, where the two sides differ by about 1e-3."""
    g = step.P.g16_arena.float()
    m = float(g[torch.isfinite(g)].abs().max()) / 65504.0
    assert lo < m < hi, f"clean step with max |g| = {m:.3f} of the fp16 range: the overflow pattern of this run is fragile"


def test_config3_reduced_overflowing_run_in_the_bench_configuration():
    """Producer-side overflow inspection + one flat update descriptor + second stream (the configuration bench.py
    times) on a run that overflows NATURALLY: the start scale 2^24 is three halvings too high, and with a growth
    interval of 3 every fourth clean step doubles the scale back into overflow.  Flags, skipped steps and the scale
    sequence must equal the free-running oracle's; a graph replay of the same run must give the eager run's bits."""
    wl = replace(I.C3_SMALL, scale=I.ScaleCfg(init_scale=2.0 ** 24, growth_interval=3))
    f = Mo.make_transformer_fwd_bwd(wl.n_layers, wl.n_seq, wl.seq_len, wl.n_heads)
    batch = wl.batch()
    n = 12
    step = St.TransformerStep(wl, prechecked=True, flat_update=True, two_streams=True)
    step.set_batch(batch)
    tr = Mo.Trainer(MIXED, _flat(wl), wl.opt, wl.scale)
    ob = Mo.island_batch(MIXED, batch)
    for k in range(n):
        tr.step(f, ob)
        before = step.P.w32_arena.clone()
        step.forward_backward()
        torch.cuda.synchronize()
        found = int(step.state().found_inf)                  # set by the gradient producers, before any inspection pass
        assert found == tr.state.history[k][1], f"step {k}: producers flagged {found}, oracle {tr.state.history[k][1]}"
        if not found:
            _assert_clean_steps_have_margin(step)
        step.optimizer()
        assert torch.equal(before, step.P.w32_arena) == bool(found), f"step {k}: skip decision"
    s = step.state()
    assert [s.hist_found_inf[i] for i in range(n)] == [1, 1, 1, 0, 0, 0, 1, 0, 0, 0, 1, 0]
    assert [s.hist_scale[i] for i in range(n)] == [h[0] for h in tr.state.history]
    assert (s.scale, s.good_steps, s.opt_step, s.skipped_steps) == (tr.state.scale, tr.state.good_steps, tr.state.opt_step, tr.state.skipped_steps)
    assert abs(float(step.loss) - tr.losses[-1]) <= 2e-3 * tr.losses[-1]
    # the default configuration (separate inspection pass, one descriptor per tensor) takes the same decisions and bits
    plain = St.TransformerStep(wl)
    plain.set_batch(batch)
    for _ in range(n):
        plain.step()
    assert torch.equal(plain.P.w32_arena, step.P.w32_arena) and torch.equal(plain.P.m_arena, step.P.m_arena)
    # ... and so does the graph replay: the skip is a device-side decision inside the captured launch sequence
    g = St.TransformerStep(wl, prechecked=True, flat_update=True, two_streams=True)
    g.set_batch(batch)
    g.step()
    graph = _graph_step(g)
    for _ in range(n - 1):
        graph.replay()
    torch.cuda.synchronize()
    sg = g.state()
    assert [sg.hist_found_inf[i] for i in range(n)] == [s.hist_found_inf[i] for i in range(n)]
    assert torch.equal(g.P.w32_arena, step.P.w32_arena) and torch.equal(g.P.w16_arena, step.P.w16_arena)


def test_config4_reduced_forced_overflow_in_the_prechecked_configuration():
    """The forced overflow of config 4 (hidden row 0 x 1e4 at step 3) with the overflow inspection left to the
    weight-gradient product's epilogue and the column sums, and one flat update descriptor."""
    wl = I.C4_SMALL
    step = St.XentStep(wl, prechecked=True, flat_update=True)
    free_running(step, wl, Mo.xent_head_fwd_bwd, None, wl.steps, batch_fn=_xent_batches(wl))
    s = step.state()
    assert [s.hist_found_inf[i] for i in range(wl.steps)] == [int(i == wl.blowup_step) for i in range(wl.steps)]
    plain = St.XentStep(wl)
    bf = _xent_batches(wl)
    for k in range(wl.steps):
        plain.set_batch(bf(k))
        plain.step()
    assert torch.equal(plain.P.w32_arena, step.P.w32_arena)


def test_config5_reduced_prechecked_configuration_matches_default():
    wl, batch = I.C5_SMALL, I.C5_SMALL.batch()
    a, b = St.LSTMStep(wl), St.LSTMStep(wl, prechecked=True, flat_update=True)
    for s_ in (a, b):
        s_.set_batch(batch)
        for _ in range(3):
            s_.step()
    assert torch.equal(a.P.w32_arena, b.P.w32_arena) and a.state().opt_step == b.state().opt_step == 3


def test_second_stream_for_weight_gradients_gives_the_same_bits():
    wl, batch = I.C3_SMALL, I.C3_SMALL.batch()
    a, b = St.TransformerStep(wl), St.TransformerStep(wl, two_streams=True)
    for s in (a, b):
        s.set_batch(batch)
        for _ in range(3):
            s.step()
    torch.cuda.synchronize()
    assert torch.equal(a.P.w32_arena, b.P.w32_arena) and torch.equal(a.P.g16_arena, b.P.g16_arena)


def test_config2_full_size():
    """Config 2 as stated: in-situ operation checks, two teacher-forced iterations, then all 50 iterations
    free-running against the oracle (Section 3.1 item 1: the scale is set for the NEXT iteration, so the sequence over
    real steps is the claim): 2^15 for steps 0-9, doubling every 10 clean steps, 2^20 after the last."""
    from test_oracle_optimizer import _golden
    wl = I.C2
    assert wl.steps == 50
    f = Mo.make_transformer_fwd_bwd(wl.n_layers, wl.n_seq, wl.seq_len, wl.n_heads)
    batch = wl.batch()
    step = St.TransformerStep(wl)
    step.set_batch(batch)
    op_level_transformer(step, wl, batch)
    teacher_forced(step, wl, f, batch, 2, grad_mode="vs_fp64")
    run = St.TransformerStep(wl, prechecked=True, flat_update=True, two_streams=True)
    run.set_batch(batch)
    free_running(run, wl, f, batch, wl.steps)
    s, g = run.state(), _golden()["c2"]
    assert [s.hist_scale[i] for i in range(wl.steps)] == g["seq"]
    assert (s.scale, s.good_steps, s.opt_step, s.skipped_steps) == (g["final"], g["good"], g["t"], g["skipped"])


# ------------------------------------------------------------------ config 4
def _xent_batches(wl):
    base = wl.batch()

    def batch_fn(k):
        b = dict(base)
        if k == wl.blowup_step:
            h = base["h"].copy()
            h[0] *= wl.blowup_factor
            b["h"] = h
        return b
    return batch_fn


def test_config4_reduced_size():
    wl = I.C4_SMALL
    step = St.XentStep(wl)
    teacher_forced(step, wl, Mo.xent_head_fwd_bwd, None, wl.steps, expect_found={wl.blowup_step}, batch_fn=_xent_batches(wl))
    step2 = St.XentStep(wl)
    free_running(step2, wl, Mo.xent_head_fwd_bwd, None, wl.steps, batch_fn=_xent_batches(wl))
    s = step2.state()
    assert [s.hist_found_inf[i] for i in range(wl.steps)] == [int(i == wl.blowup_step) for i in range(wl.steps)]


# ------------------------------------------------------------------ config 5
@pytest.mark.parametrize("persistent", [True, False])
def test_config5_reduced_size(persistent):
    """Both launch plans of the LSTM stack: one recurrent kernel per layer and direction, and step by step."""
    wl = I.C5_SMALL
    f = Mo.make_lstm_fwd_bwd(wl.n_layers)
    batch = wl.batch()
    step = St.LSTMStep(wl, persistent=persistent)
    assert step.persistent == persistent
    step.set_batch(batch)
    teacher_forced(step, wl, f, batch, 4)
    step2 = St.LSTMStep(wl, persistent=persistent)
    step2.set_batch(batch)
    free_running(step2, wl, f, batch, wl.steps)
    assert step.recurrent_kernels_ok() and step2.recurrent_kernels_ok()


# ------------------------------------------------------------------ full sizes, in the configuration bench.py times
def test_config3_full_size_bench_configuration():
    """Config 3 at full size exactly as bench.py launches it (producer-side overflow inspection, one flat update
    descriptor, HIP-graph replay): every operation of the first and last layer checked in situ against the oracle,
    then graph replays against eager execution, bit for bit."""
    wl = I.C3
    batch = wl.batch()
    step = St.TransformerStep(wl, prechecked=True, flat_update=True)
    step.set_batch(batch)
    worst = op_level_transformer(step, wl, batch)              # every operation of all six layers
    print(f"config 3 full size: worst in-situ op error {worst:.2e}", flush=True)
    # the optimizer wrapper at 75.6 M parameters against the oracle on the GPU's own gradients
    before = _snapshot(step)
    s0 = step.state()
    g_gpu = {n: np32(step.P.g16[n]) for n in step.P.names}
    step.optimizer()
    after = _snapshot(step)
    ost = O.ScaleState(scale=float(s0.scale), growth_interval=s0.growth_interval, opt_step=s0.opt_step)
    for n in ("l0.wqkv", "l3.w1", "l5.w2", "l5.ln2_g", "l2.b1"):
        t = [dict(g16=g_gpu[n], w32=before["w32"][n].copy(), w16=before["w16"][n].copy(), m=before["m"][n].copy(), v=before["v"][n].copy())]
        assert O.unscale_check_update(MIXED, t, wl.opt, ost) == 0
        assert rel_fro(after["w32"][n], t[0]["w32"]) <= MASTER_TOL and rel_fro(after["m"][n], t[0]["m"]) <= MASTER_TOL
        assert np.array_equal(half_bits(after["w16"][n]), half_bits(MIXED.store(after["w32"][n])))
    # graph replay == eager, several replays with eager work and synchronisation between them; the replayed step is
    # the two-stream one bench.py times (weight-gradient launch and bias-gradient column sums on a second stream),
    # the eager one runs on a single stream: the bits must not depend on either
    eager = St.TransformerStep(wl, prechecked=True, flat_update=True)
    eager.set_batch(batch)
    eager.step()
    assert torch.equal(step.P.w32_arena, eager.P.w32_arena)
    two = St.TransformerStep(wl, prechecked=True, flat_update=True, two_streams=True)
    two.set_batch(batch)
    two.step()
    graph = _graph_step(two)                      # capture = step 2 is recorded, not run
    for _ in range(3):
        graph.replay()
        eager.step()
        torch.cuda.synchronize()
        assert float(two.loss) == float(eager.loss)
        assert torch.equal(two.P.w32_arena, eager.P.w32_arena) and torch.equal(two.P.w16_arena, eager.P.w16_arena)
    s = two.state()
    assert (s.opt_step, s.skipped_steps, s.scale) == (4, 0, 2.0 ** 15)


def test_config3_full_size_three_teacher_forced_steps():
    """Config 3 at full size in the bench configuration, three iterations against the oracle: loss, whole-network
    gradients (as close to the fp64 definition as the oracle's, see teacher_forced), the optimizer wrapper on EVERY
    tensor (masters and moments <= 1e-5, fp16 copies exact) and every field of the scale state."""
    wl = I.C3
    f = Mo.make_transformer_fwd_bwd(wl.n_layers, wl.n_seq, wl.seq_len, wl.n_heads)
    batch = wl.batch()
    step = St.TransformerStep(wl, prechecked=True, flat_update=True, two_streams=True)
    step.set_batch(batch)
    worst = teacher_forced(step, wl, f, batch, 3, grad_mode="vs_fp64", progress="config 3 full size")
    print(f"config 3 full size, 3 teacher-forced steps: worst {worst}", flush=True)
    s = step.state()
    assert (s.opt_step, s.skipped_steps, s.scale, s.good_steps) == (3, 0, 2.0 ** 15, 3)


def test_config3_full_size_scale_sequence_over_growth_interval():
    """120 iterations on the GPU; the recorded overflow flags replayed through the oracle's state machine must give
    the recorded scale sequence (growth at iteration 100), and no iteration may overflow."""
    wl = replace(I.C3, steps=120)
    step = St.TransformerStep(wl, prechecked=True, flat_update=True, two_streams=True)
    step.set_batch(wl.batch())
    step.step()
    graph = _graph_step(step)
    for _ in range(wl.steps - 1):
        graph.replay()
    s = step.state()
    ost = O.ScaleState(scale=float(wl.scale.init_scale), growth_interval=wl.scale.growth_interval)
    for i in range(wl.steps):
        O.loss_scale_update(ost, int(s.hist_found_inf[i]))
    assert [s.hist_scale[i] for i in range(wl.steps)] == [h[0] for h in ost.history]
    assert [s.hist_scale[i] for i in range(wl.steps)] == [2.0 ** 15] * 100 + [2.0 ** 16] * 20
    assert (s.scale, s.good_steps, s.opt_step, s.skipped_steps) == (ost.scale, ost.good_steps, 120, 0)
    assert np.isfinite(float(step.loss))


def test_config4_full_size():
    """Vocabulary projection + cross-entropy at 8192 x 32768: steps 0-4 free-running against the oracle (overflow
    forced at step 3 by the x1e4 hidden row, scale halved for step 4), then the rest on the GPU alone with the flag
    stream replayed through the oracle's state machine (golden sequence c4)."""
    from test_oracle_optimizer import _golden
    wl = I.C4
    bf = _xent_batches(wl)
    step = St.XentStep(wl)
    tr = Mo.Trainer(MIXED, wl.masters(), wl.opt, wl.scale)
    for k in range(5):
        b = bf(k)
        step.set_batch(b)
        keep = {}
        ob = Mo.island_batch(MIXED, b)
        w_before = {n: np32(step.P.w16[n]) for n in step.P.names}
        step.forward_backward()
        loss_ref, g_ref = Mo.xent_head_fwd_bwd(MIXED, w_before, ob, float(step.state().scale), keep=keep)
        bad = O.has_nonfinite(MIXED, list(g_ref.values()))
        assert bad == (k == wl.blowup_step)
        assert abs(float(step.loss) - float(loss_ref)) <= 2e-4 * abs(float(loss_ref))
        if not bad:
            for n in step.P.names:
                assert rel_fro(np32(step.P.g16[n]), g_ref[n]) <= GRAD_TOL, (k, n)
            assert rel_fro(np32(step.dh), keep["dh"]) <= GRAD_TOL
        else:
            assert O.has_nonfinite(MIXED, [np32(step.P.g16["w"])])
        step.optimizer()
        print(f"config 4 step {k}: loss {float(step.loss):.4f} overflow={bad}", flush=True)
    for k in range(5, wl.steps):
        step.set_batch(bf(k)) if k == 5 else None
        step.step()
    s, g = step.state(), _golden()["c4"]
    assert [s.hist_scale[i] for i in range(wl.steps)] == g["seq"]
    assert [s.hist_found_inf[i] for i in range(wl.steps)] == [int(i in g["ovf"]) for i in range(wl.steps)]
    assert (s.scale, s.good_steps, s.opt_step, s.skipped_steps) == (g["final"], g["good"], g["t"], g["skipped"])


def test_config5_full_size():
    """GNMT-like LSTM stack at full size: one teacher-forced iteration against the oracle, then 20 iterations on the
    GPU with the scale sequence checked against the hand-derived one (c5)."""
    from test_oracle_optimizer import _golden
    wl = I.C5
    f = Mo.make_lstm_fwd_bwd(wl.n_layers)
    batch = wl.batch()
    step = St.LSTMStep(wl)
    step.set_batch(batch)
    # 4 layers x 50 time steps of recurrence compound fp16 roundings to ~1e-3 at the bottom layer, for the
    # oracle as much as for the GPU: the whole-network check is "as close to fp64 as the oracle" (the
    # reduced-size run above holds 1e-3 directly, and the cell / gate kernels are checked in isolation).
    assert step.persistent
    teacher_forced(step, wl, f, batch, 1, grad_mode="vs_fp64")
    graph = _graph_step(step)                   # iteration 2 is recorded, then replayed: persistent kernels inside a HIP graph
    for _ in range(wl.steps - 1):
        graph.replay()
    assert step.recurrent_kernels_ok()
    s, g = step.state(), _golden()["c5"]
    assert [s.hist_scale[i] for i in range(wl.steps)] == g["seq"]
    assert (s.scale, s.good_steps, s.opt_step, s.skipped_steps) == (g["final"], g["good"], g["t"], g["skipped"])
    assert np.isfinite(float(step.loss))
    # the step-by-step plan at full size gives the same training run to within summation order
    slow = St.LSTMStep(wl, persistent=False)
    slow.set_batch(batch)
    for _ in range(3):
        slow.step()
    fast = St.LSTMStep(wl)
    fast.set_batch(batch)
    for _ in range(3):
        fast.step()
    assert abs(float(slow.loss) - float(fast.loss)) <= 1e-4 * float(fast.loss)
    for n in fast.P.names:
        assert rel_fro(np32(fast.P.g16[n]), np32(slow.P.g16[n])) <= 2e-2, n   # (200 steps deep: see teacher_forced "vs_fp64")


def test_graph_replay_matches_eager_small():
    """HIP-graph capture of a whole iteration (no memset nodes: fills are kernels) replays bit-identically, with
    eager work and synchronisation between replays."""
    wl, batch = I.C3_SMALL, I.C3_SMALL.batch()
    a, b = St.TransformerStep(wl), St.TransformerStep(wl)
    for s in (a, b):
        s.set_batch(batch)
        s.step()
    graph = _graph_step(a)
    for _ in range(4):
        graph.replay()
        b.step()
        torch.cuda.synchronize()
        assert float(a.loss) == float(b.loss) and torch.equal(a.P.w32_arena, b.P.w32_arena)
    assert a.state().opt_step == b.state().opt_step == 5


def test_workload_runner_command_line(capsys):
    """python -m paper_1805_10387_amd.steps <n>: one JSON line per run, eager and as a graph replay."""
    import json
    St._main(["1", "--steps", "3", "--warmup", "1"])
    St._main(["2", "--steps", "2", "--warmup", "1", "--graph"])
    lines = [json.loads(l) for l in capsys.readouterr().out.strip().splitlines() if l.startswith("{")]
    assert [l["config"] for l in lines] == [1, 2] and lines[1]["launch"] == "HIP graph replay"
    assert all(l["ms_per_step"] > 0 and np.isfinite(l["loss"]) and l["skipped"] == 0 for l in lines)
    assert lines[0]["opt_steps"] == 4 and lines[1]["opt_steps"] == 4          # warm-up + capture/first replay + timed
