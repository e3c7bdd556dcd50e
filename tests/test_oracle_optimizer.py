"""Pins for the oracle's optimizer wrapper, scale policy and the method's invariants (CPU only)."""
import os

import numpy as np
import pytest

import mp_inputs as I
from oracle import MIXED, FP32, FP64
from oracle import models as Mo
from oracle.numerics import half_bits
from oracle.optimizer import ScaleState, loss_scale_update, unscale_check_update, has_nonfinite
from refbits import f32_to_f16_bits

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "scale_sequences.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        name, cfg, ovf, runs, final = [s.strip() for s in line.split("|")]
        s0, n, steps = [int(t) for t in cfg.split()]
        seq = [2.0 ** int(r.split(":")[0]) for r in runs.split() for _ in range(int(r.split(":")[1]))]
        fl, good, t, skipped = [int(t) for t in final.split()]
        out[name] = dict(s0=2.0 ** s0, n=n, steps=steps, ovf={int(t) for t in ovf.split()}, seq=seq,
                         final=2.0 ** fl, good=good, t=t, skipped=skipped)
    return out


@pytest.mark.parametrize("name", ["c1", "c2", "c4", "c5", "floor"])
def test_backoff_state_machine_against_hand_derived_sequences(name):
    g = _golden()[name]
    st = ScaleState(mode="backoff", scale=g["s0"], growth_interval=g["n"])
    for step in range(g["steps"]):
        loss_scale_update(st, int(step in g["ovf"]))
    assert [h[0] for h in st.history] == g["seq"]
    assert [h[1] for h in st.history] == [int(s in g["ovf"]) for s in range(g["steps"])]
    assert (st.scale, st.good_steps, st.opt_step, st.skipped_steps) == (g["final"], g["good"], g["t"], g["skipped"])


def test_scale_clamps_at_ceiling_and_static_mode_never_moves():
    st = ScaleState(mode="backoff", scale=2.0 ** 23, growth_interval=1, max_scale=2.0 ** 24)
    for _ in range(3):
        loss_scale_update(st, 0)
    assert st.scale == 2.0 ** 24
    st = ScaleState(mode="static", scale=10.0, growth_interval=1)
    for f in (0, 1, 0, 0):
        loss_scale_update(st, f)
    assert st.scale == 10.0 and st.skipped_steps == 1 and st.opt_step == 3


def _tensor(P, w, g, adam=True):
    w32 = P.island(w).copy()
    return dict(g16=P.store(g), w32=w32, w16=P.store(w32), m=np.zeros_like(w32), v=np.zeros_like(w32))


def test_adam_first_step_closed_form_and_fp16_copy():
    rng = np.random.default_rng(20)
    w = rng.standard_normal(5000).astype(np.float32) * 0.05
    g = rng.standard_normal(5000).astype(np.float32) * 3.0
    S = 2.0 ** 7
    t = _tensor(MIXED, w, g * S)
    st = ScaleState(scale=S)
    opt = I.OptCfg(kind="adam", lr=1e-3)
    assert unscale_check_update(MIXED, [t], opt, st) == 0
    gq = t["g16"].astype(np.float64) / S
    # step 1 of Adam: m_hat = g, v_hat = g^2  =>  dw = -lr g / (|g| + eps)
    expect = w.astype(np.float64) - 1e-3 * gq / (np.abs(gq) + 1e-8)
    assert np.max(np.abs(t["w32"] - expect)) < 2e-7 * 0.3
    assert np.allclose(t["m"], 0.1 * gq, rtol=1e-6) and np.allclose(t["v"], 0.001 * gq * gq, rtol=1e-5)
    assert np.array_equal(half_bits(t["w16"]), f32_to_f16_bits(t["w32"]))


def test_adam_matches_torch_adam_over_steps():
    import torch
    rng = np.random.default_rng(21)
    w = rng.standard_normal(300) * 0.1
    t = _tensor(FP64, w, np.zeros(300))
    st = ScaleState(scale=4.0)
    opt = I.OptCfg(kind="adam", lr=1e-2)
    tw = torch.from_numpy(w.copy()).requires_grad_()
    topt = torch.optim.Adam([tw], lr=1e-2, betas=(0.9, 0.999), eps=1e-8)
    for k in range(7):
        g = rng.standard_normal(300)
        t["g16"] = g * 4.0
        unscale_check_update(FP64, [t], opt, st)
        loss_scale_update(st, 0)
        tw.grad = torch.from_numpy(g.copy())
        topt.step()
    assert np.allclose(t["w32"], tw.detach().numpy(), rtol=0, atol=1e-13)


def test_sgd_and_weight_decay_on_master():
    w = np.array([0.5, -0.25, 1e-3], dtype=np.float32)
    g = np.array([2.0, -4.0, 8.0], dtype=np.float32)
    t = _tensor(MIXED, w, g)
    st = ScaleState(scale=2.0)
    unscale_check_update(MIXED, [t], I.OptCfg(kind="sgd", lr=0.125), st)
    assert np.array_equal(t["w32"], np.float32(w - 0.125 * g / 2))
    # Section 3.3: the regulariser's gradient wd*w is formed on the fp32 copy and added after unscaling;
    # wd*w = 1e-5 * 1e-3 = 1e-8 is below the smallest fp16 subnormal (6e-8) yet moves the master.
    t2 = _tensor(MIXED, w, np.zeros(3))
    unscale_check_update(MIXED, [t2], I.OptCfg(kind="sgd", lr=1.0, weight_decay=1e-5), st)
    assert np.allclose(t2["w32"], w * (1 - 1e-5), rtol=1e-7) and t2["w32"][2] != w[2]
    assert float(MIXED.store(np.float32(1e-8))) == 0.0


@pytest.mark.parametrize("bad", [np.inf, -np.inf, np.nan])
@pytest.mark.parametrize("where", [0, 77, 199])
def test_skip_leaves_every_buffer_untouched(bad, where):
    rng = np.random.default_rng(22)
    ts = [_tensor(MIXED, rng.standard_normal(100) * 0.1, rng.standard_normal(100)) for _ in range(2)]
    for t in ts:                       # give the moments a history
        t["m"] += 0.01
        t["v"] += 0.02
    ts[where // 100]["g16"][where % 100] = bad
    before = [{k: v.copy() for k, v in t.items()} for t in ts]
    st = ScaleState(scale=2.0 ** 15, growth_interval=3, good_steps=2, opt_step=5)
    found = unscale_check_update(MIXED, ts, I.OptCfg(), st)
    loss_scale_update(st, found)
    assert found == 1
    for t, b in zip(ts, before):
        for k in ("w32", "w16", "m", "v"):
            assert t[k].tobytes() == b[k].tobytes()
    assert (st.scale, st.good_steps, st.opt_step, st.skipped_steps) == (2.0 ** 14, 0, 5, 1)


def test_nonfinite_test_is_on_the_half_encoding():
    assert not has_nonfinite(MIXED, [np.array([65504.0, -65504.0, 0.0, 6e-8], np.float32)])
    assert has_nonfinite(MIXED, [np.zeros(3, np.float32), np.array([1.0, np.inf], np.float32)])
    assert has_nonfinite(MIXED, [np.array([np.nan], np.float32)])


def test_master_copy_accumulates_updates_fp16_would_lose():
    # Section 3.1 item 2: an update below half an fp16 ulp of the weight is kept by the fp32 master.
    w = np.array([1.0], dtype=np.float32)               # ulp16(1.0) = 2^-10
    g = np.array([1.0], dtype=np.float32)
    t = _tensor(MIXED, w, g)
    st = ScaleState(scale=1.0)
    opt = I.OptCfg(kind="sgd", lr=2.0 ** -13)           # each step moves the master by 2^-13 = ulp/8
    w16_only = MIXED.store(w)
    flips = []
    for k in range(8):
        unscale_check_update(MIXED, [t], opt, st)
        w16_only = MIXED.store(w16_only - np.float32(2.0 ** -13) * g)   # fp16-only training: stuck
        flips.append(float(t["w16"][0]))
    assert float(w16_only[0]) == 1.0
    assert float(t["w32"][0]) == 1.0 - 8 * 2.0 ** -13
    assert flips[-1] == 1.0 - 2.0 ** -10 and flips[0] == 1.0


def _run_c1(P, wl, scale_cfg=None, steps=None, inject=True):
    tr = Mo.Trainer(P, wl.masters(), wl.opt, scale_cfg or wl.scale)
    batch = Mo.island_batch(P, wl.batch())
    for step in range(steps or wl.steps):
        inj = None
        if inject and step == wl.inject_step:
            def inj(grads):
                grads["w2"].reshape(-1)[0] = np.inf
        tr.step(Mo.mlp_fwd_bwd, batch, inj)
    return tr


def test_config1_end_to_end_scale_sequence_and_learning():
    g = _golden()["c1"]
    tr = _run_c1(MIXED, I.C1)
    assert [h[0] for h in tr.state.history] == g["seq"]
    assert [h[1] for h in tr.state.history] == [int(s in g["ovf"]) for s in range(20)]
    assert (tr.state.scale, tr.state.good_steps, tr.state.opt_step, tr.state.skipped_steps) == (g["final"], g["good"], g["t"], g["skipped"])
    assert tr.losses[-1] < tr.losses[0]
    assert tr.losses[7] == tr.losses[8]                  # step 7 was skipped: same weights at step 8


def test_mixed_loss_curve_matches_fp32(monkeypatch=None):
    # Section 5 / Figure 3 of the paper: mixed-precision loss curves track FP32 closely.
    a = _run_c1(MIXED, I.C1, inject=False)
    b = _run_c1(FP32, I.C1, inject=False)
    assert abs(a.losses[-1] - b.losses[-1]) / b.losses[-1] < 1e-2
    assert np.max(np.abs(np.array(a.losses) - np.array(b.losses)) / np.array(b.losses)) < 1e-2


def test_loss_scaling_commutes_exactly_when_nothing_leaves_normal_range():
    # Backward is linear in the seed gradient and S is a power of two, so every rounding commutes with
    # the scaling as long as no value is subnormal or overflows: gradients at scale 2^8, divided by 2^4,
    # equal gradients at scale 2^4 bit for bit.
    wl = I.MLPWorkload(rows=4, d_in=16, d_hidden=32, d_out=8)
    w = {k: MIXED.store(v * 10) for k, v in wl.masters().items()}
    b = wl.batch()
    b["target"] = b["target"] * 50
    b = Mo.island_batch(MIXED, b)
    ka, kb = {}, {}
    _, ga = Mo.mlp_fwd_bwd(MIXED, w, b, 2.0 ** 4, keep=ka)
    _, gb = Mo.mlp_fwd_bwd(MIXED, w, b, 2.0 ** 8, keep=kb)
    allv = np.concatenate([np.abs(v).ravel() for v in list(ga.values()) + [ka["dy"], ka["dpre"], ka["dx"]]])
    assert allv[allv > 0].min() >= 2.0 ** -14 and allv.max() * 16 < 65504     # precondition of the claim
    for k in ga:
        assert np.array_equal(ga[k] * np.float32(16), gb[k]), k


def test_loss_scaling_rescues_underflowing_gradients():
    # With scale 1 the seed gradient 2(y-t)/numel ~ 1e-5 of a 512-row batch sits in the fp16 subnormal range
    # and the hidden-layer gradient ~1e-7 mostly flushes to zero; with scale 2^10 the unscaled gradients
    # are far closer to the fp64 truth.
    from dataclasses import replace
    wl = replace(I.C1, rows=512)
    w = {k: MIXED.store(v) for k, v in wl.masters().items()}
    b = Mo.island_batch(MIXED, wl.batch())
    _, g64 = Mo.mlp_fwd_bwd(FP64, {k: v.astype(np.float64) for k, v in w.items()},
                            {k: v.astype(np.float64) for k, v in b.items()}, 1.0)
    _, g1 = Mo.mlp_fwd_bwd(MIXED, w, b, 1.0)
    _, gs = Mo.mlp_fwd_bwd(MIXED, w, b, 2.0 ** 10)
    e1 = np.linalg.norm(g1["w1"] - g64["w1"]) / np.linalg.norm(g64["w1"])
    es = np.linalg.norm(gs["w1"] / 1024.0 - g64["w1"]) / np.linalg.norm(g64["w1"])
    assert es < 1e-3 and e1 > 5 * es
    tiny = np.float32(2.5e-8)                      # a gradient value below half the smallest subnormal
    assert float(MIXED.store(tiny)) == 0.0 and float(MIXED.store(tiny * 1024)) != 0.0
