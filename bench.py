#!/usr/bin/env python3
"""Throughput of the mixed-precision training step (config 3: Transformer-big layer stack) on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W]

One "step" is the whole hot path over one synthetic batch already resident in HBM: 6 encoder layers
forward, MSE loss with the loss-scaled seed gradient, backward (all dX and dW contractions), the fused
unscale / overflow-check / Adam update of the fp32 masters with the fp16 re-cast, and the loss-scale
update.  The step is captured once in a HIP graph and replayed K times between two events.

Prints ONE JSON line with tokens/s plus
  roofline        : the dense fp16 MFMA contractions of the step (per-launch flops / per-launch time
                    measured with HIP events on the launch stream) against the fp16 dense peak
  roofline_update : the fused optimizer kernel against peak HBM bandwidth
  cpu_baseline    : the NumPy oracle timed on this host on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time
from dataclasses import replace

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP16_TFLOPS = 2500.0   # MI355X dense fp16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "gemm_update_config3_hbm_traffic.txt")


def traffic_from_summary():
    """HBM bytes per launch (FETCH_SIZE + WRITE_SIZE, each scaled by what the same counter reads for a 256 MiB copy) as
    the last counter runs of this script left them in profiles/ (written by `python -m paper_1805_10387_amd.profile_summary
    traffic ...`, whose command lines are in that file).  None when the summary is missing: the value is never typed in."""
    out = {"gemm": None, "update": None}
    try:
        for line in open(TRAFFIC_SUMMARY):
            for key in out:
                tag = f"{key}_traffic_bytes_per_launch ="
                if line.strip().startswith(tag):
                    out[key] = int(float(line.split("=")[1].split()[0]))
    except OSError:
        pass
    return out


def _time_calls(torch, fn, reps):
    """Average duration (s) of fn() launched reps times back to back on the current stream."""
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / reps


def gemm_roofline(torch, B, step, reps=20):
    """Time each distinct dense-contraction launch of one layer in isolation (same descriptors, same buffers as
    the step uses) and aggregate: algorithmic flops = 2 M N K per product."""
    wl, w, g, a = step.wl, step.P.w16, step.P.g16, step.act[0]
    tb = step.tmp[0]
    dqkv, dz1, dz2, df = tb["dqkv"], tb["dz1"], tb["dz2"], tb["df"]
    T, d, f = wl.tokens, wl.d_model, wl.d_ff
    x, ws, st = step.x0, step.ws, step.st
    calls = {
        "fwd_qkv": (2.0 * T * 3 * d * d, lambda: B.mp_gemm_fwd(step.d_qkv, x, w["l0.wqkv"], w["l0.bqkv"], None, a["qkv"])),
        "fwd_o": (2.0 * T * d * d, lambda: B.mp_gemm_fwd(step.d_o, a["ctx"], w["l0.wo"], w["l0.bo"], None, a["a"])),
        "fwd_ffn1": (2.0 * T * f * d, lambda: B.mp_gemm_fwd(step.d_f1, a["y1"], w["l0.w1"], w["l0.b1"], None, a["f"])),
        "fwd_ffn2": (2.0 * T * f * d, lambda: B.mp_gemm_fwd(step.d_f2, a["f"], w["l0.w2"], w["l0.b2"], None, a["g"])),
        "dx_qkv": (2.0 * T * 3 * d * d, lambda: B.mp_gemm_bwd_dx(step.d_qkv, dqkv, w["l0.wqkv"], step.gbuf[1], add=dz1, ld_aux=d)),
        "dx_o": (2.0 * T * d * d, lambda: B.mp_gemm_bwd_dx(step.d_o, dz1, w["l0.wo"], step.dctx)),
        "dx_ffn1": (2.0 * T * f * d, lambda: B.mp_gemm_bwd_dx(step.d_f1, df, w["l0.w1"], step.dy1, add=dz2, ld_aux=d)),
        "dx_ffn2": (2.0 * T * f * d, lambda: B.mp_gemm_bwd_dx(step.d_f2, dz2, w["l0.w2"], df, relu_src=a["f"], ld_aux=f)),
    }
    if step.grouped_dw:
        grp = B.gemm_group([(step.d_f2, dz2, a["f"], g["l0.w2"]), (step.d_f1, df, a["y1"], g["l0.w1"], g["l0.b1"]),
                            (step.d_qkv, dqkv, x, g["l0.wqkv"], g["l0.bqkv"]), (step.d_o, dz1, a["ctx"], g["l0.wo"])])
        calls["dw_grouped(qkv,o,ffn1,ffn2 + bias gradients of ffn1, qkv)"] = (2.0 * T * (4 * d * d + 2 * f * d), lambda: B.mp_gemm_bwd_dw_grouped(grp, st))
    else:
        calls.update({
            "dw_qkv": (2.0 * T * 3 * d * d, lambda: B.mp_gemm_bwd_dw(step.d_qkv, dqkv, x, g["l0.wqkv"], None, st, ws)),
            "dw_o": (2.0 * T * d * d, lambda: B.mp_gemm_bwd_dw(step.d_o, dz1, a["ctx"], g["l0.wo"], None, st, ws)),
            "dw_ffn1": (2.0 * T * f * d, lambda: B.mp_gemm_bwd_dw(step.d_f1, df, a["y1"], g["l0.w1"], None, st, ws)),
            "dw_ffn2": (2.0 * T * f * d, lambda: B.mp_gemm_bwd_dw(step.d_f2, dz2, a["f"], g["l0.w2"], None, st, ws)),
        })
    per, flops, secs = {}, 0.0, 0.0
    for name, (fl, fn) in calls.items():
        t = _time_calls(torch, fn, reps)
        per[name] = {"us": round(t * 1e6, 2), "tflops": round(fl / t * 1e-12, 1)}
        flops += fl
        secs += t
    return flops, secs, per


class GemmTimer:
    """Brackets every dense-contraction call the step makes (mp_gemm_fwd / mp_gemm_bwd_dx / mp_gemm_bwd_dw)
    with a pair of events on the launch stream while the step runs eagerly, so each launch is timed where it
    runs in the step: same operands, same cache state, same neighbours.  flops = 2 M N K x batches."""

    NAMES = ("mp_gemm_fwd", "mp_gemm_bwd_dx", "mp_gemm_bwd_dw", "mp_gemm_bwd_dw_grouped")

    def __init__(self, torch, B):
        self.torch, self.B, self.saved, self.rec = torch, B, {}, []

    def __enter__(self):
        for name in self.NAMES:
            fn = getattr(self.B, name)
            self.saved[name] = fn

            def timed(desc, *a, _fn=fn, _name=name, **kw):
                e0, e1 = self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True)
                e0.record()
                r = _fn(desc, *a, **kw)
                e1.record()
                # (the grouped entry point takes an array of items, each with its own descriptor)
                descs = [it.desc for it in desc] if _name == "mp_gemm_bwd_dw_grouped" else [desc]
                fl = sum(2.0 * q.M * q.N * q.K * max(q.batch_outer, 1) * max(q.batch_inner, 1) for q in descs)
                byts = sum(2.0 * (q.M * q.K + q.K * q.N + q.M * q.N) * max(q.batch_outer, 1) * max(q.batch_inner, 1) for q in descs)
                # an empty bracket right behind it: what two event records cost on this stream with nothing between
                z0, z1 = self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True)
                z0.record()
                z1.record()
                self.rec.append((e0, e1, fl, byts, z0, z1))
                return r
            setattr(self.B, name, timed)
        return self

    def __exit__(self, *exc):
        for name, fn in self.saved.items():
            setattr(self.B, name, fn)

    def totals(self):
        self.torch.cuda.synchronize()
        raw = sum(r[0].elapsed_time(r[1]) for r in self.rec) * 1e-3
        empty = sum(r[4].elapsed_time(r[5]) for r in self.rec) * 1e-3
        return len(self.rec), sum(r[2] for r in self.rec), sum(r[3] for r in self.rec), raw, empty


def _host_cores():
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


def _time_oracle(wl, iterations, threads=None):
    """Seconds per complete oracle iteration (forward, loss, backward, Adam on masters) of a Transformer workload."""
    from threadpoolctl import threadpool_info, threadpool_limits
    from oracle import MIXED
    from oracle import models as Mo
    masters = Mo.flatten_layers(wl.masters())
    tr = Mo.Trainer(MIXED, masters, wl.opt, wl.scale)
    f = Mo.make_transformer_fwd_bwd(wl.n_layers, wl.n_seq, wl.seq_len, wl.n_heads)
    batch = Mo.island_batch(MIXED, wl.batch())
    times = []
    ctx = threadpool_limits(limits=threads) if threads else None
    try:
        for _ in range(iterations):
            t0 = time.perf_counter()
            tr.step(f, batch)
            times.append(time.perf_counter() - t0)
        used = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    finally:
        if ctx is not None:
            ctx.restore_original_limits()
    return min(times), times, int(used)


def cpu_baseline(wl, c2, iterations=2):
    """The oracle, as it stands, on the FULL config-3 workload (6 layers, all 64 sequences = 8192 tokens): complete
    iterations, best of `iterations`; plus one single-thread figure on config 2 (one layer, 4096 tokens)."""
    best, times, used = _time_oracle(wl, iterations)
    c2_best, c2_times, _ = _time_oracle(c2, 2, threads=1)
    return {"value": wl.tokens / best, "unit": "tokens/s", "cores": used, "host_cores": _host_cores(), "kind": "oracle",
            "blas_threads": used,
            "sample": f"full workload: {wl.n_layers} layers x {wl.n_seq} sequences x {wl.seq_len} tokens, {len(times)} complete "
                      f"iterations ({', '.join(f'{t:.1f}' for t in times)} s), best {best:.2f} s/iteration; NumPy with its BLAS on "
                      f"{used} threads of {_host_cores()} host cores",
            "config2_single_core": {"value": c2.tokens / c2_best, "unit": "tokens/s", "cores": 1,
                                    "sample": f"config 2 (1 layer, {c2.tokens} tokens), 2 complete iterations, best {c2_best:.2f} s"}}


def glue_roofline(torch, B, step, I):
    """The bandwidth-bound kernels of the step, each alone and back to back on its own buffers: algorithmic bytes (every
    stored tensor read / written once) over time, against 8 TB/s."""
    wl, a, w = step.wl, step.act[0], step.P.w16
    T, d, h, S, NB = wl.tokens, wl.d_model, wl.n_heads, wl.seq_len, wl.n_seq
    tb = step.tmp[0]
    st = step.st
    e2 = 2.0  # bytes per fp16 element
    P_bytes = NB * h * S * S * e2
    calls = {
        "attention_fwd": (T * 3 * d * e2 + P_bytes + T * d * e2,
                          lambda: B.mp_attention_fwd(NB, h, S, d // h, a["qkv"], 3 * d, step.alpha, a["p"], a["ctx"], d)),
        "attention_bwd": (T * 3 * d * e2 + P_bytes + T * d * e2 + T * 3 * d * e2,
                          lambda: B.mp_attention_bwd(NB, h, S, d // h, a["qkv"], 3 * d, step.alpha, a["p"], step.dctx, d, tb["dqkv"], 3 * d)),
        "layernorm_fwd": (3 * T * d * e2 + 8.0 * T,
                          lambda: B.mp_layernorm_fwd(T, d, step.x0, a["a"], w["l0.ln1_g"], w["l0.ln1_b"], 1e-5, a["y1"], a["mean1"], a["rstd1"])),
        "layernorm_bwd": (4 * T * d * e2 + 8.0 * T,
                          lambda: B.mp_layernorm_bwd(T, d, step.dy1, step.x0, a["a"], w["l0.ln1_g"], a["mean1"], a["rstd1"], tb["dz1"],
                                                     step.P.g16["l0.ln1_g"], step.P.g16["l0.ln1_b"], st, step.ws, dz_colsum=step.P.g16["l0.bo"])),
    }
    # softmax cross-entropy at config 4's size (8192 x 32768 logits, in place): not part of this step, timed for the record
    c4 = I.C4
    logits = torch.randn(c4.tokens, c4.vocab, device="cuda", dtype=torch.float16)
    targets = torch.randint(0, c4.vocab, (c4.tokens,), device="cuda", dtype=torch.int32)
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    ws = torch.empty(B.mp_loss_workspace_bytes(c4.tokens, c4.vocab) // 4 + 64, dtype=torch.float32, device="cuda")
    calls["softmax_xent (config 4 size)"] = (2.0 * c4.tokens * c4.vocab * e2,
                                             lambda: B.mp_softmax_xent_scaled(c4.tokens, c4.vocab, logits, c4.vocab, targets, st, loss, logits, ws))
    out = {}
    for name, (nbytes, fn) in calls.items():
        t = _time_calls(torch, fn, 20)
        out[name] = {"bytes": nbytes, "us": round(t * 1e6, 2), "GB/s": round(nbytes / t * 1e-9, 1),
                     "frac": round(nbytes / t * 1e-9 / PEAK_HBM_GBS, 3)}
    del logits
    return out


def sclk_under_load(torch, run, seconds=1.5):
    """Shader clock (MHz) that rocm-smi reports while the step replays: the chip lowers it under matrix-core load
    according to the power the operand values draw, which moves the real ceiling below the datasheet peak."""
    import json as _json
    import subprocess
    import threading
    vals, stop = [], [False]

    def sampler():
        while not stop[0]:
            try:
                o = subprocess.run(["rocm-smi", "--showclocks", "--json"], capture_output=True, text=True, timeout=5).stdout
                c = _json.loads(o)["card0"]
                for k, v in c.items():
                    if k.startswith("sclk clock speed"):
                        vals.append(int("".join(ch for ch in v if ch.isdigit())))
            except Exception:
                return
            time.sleep(0.1)

    th = threading.Thread(target=sampler)
    th.start()
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(20):
            run()
        torch.cuda.synchronize()
    stop[0] = True
    th.join()
    vals = sorted(vals[1:]) if len(vals) > 2 else sorted(vals)
    return vals[len(vals) // 2] if vals else None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=120, help="timed steps per repeat")
    ap.add_argument("--repeats", type=int, default=5, help="timed repeats of --steps steps; the median is reported")
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-graph", action="store_true", help="launch every kernel from Python instead of replaying a HIP graph")
    ap.add_argument("--one-stream", action="store_true",
                    help="keep the grouped weight-gradient launch of each layer on the main stream")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-iterations", type=int, default=2, help="complete oracle iterations of the full workload")
    ap.add_argument("--insitu-steps", type=int, default=3, help="eager steps whose contractions are timed one by one")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1. "
              "Sharding the step over several GPUs (one gradient exchange before the update) is designed, not built.", file=sys.stderr)
        sys.exit(2)

    import torch
    import mp_inputs as I
    import paper_1805_10387_amd as mp
    from paper_1805_10387_amd import binding as B
    from paper_1805_10387_amd import steps as St

    torch.cuda.set_device(0)
    wl = I.C3
    step = St.TransformerStep(wl, prechecked=True, flat_update=True, two_streams=not args.one_stream)
    step.set_batch(wl.batch())
    for _ in range(max(args.warmup, 1)):
        step.step()
    torch.cuda.synchronize()

    if args.no_graph:
        run = step.step
    else:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step.step()
        run = graph.replay
        run()
    torch.cuda.synchronize()
    # timing protocol: `repeats` times exactly `steps` steps between two events on the stream, no host sync inside;
    # the median repeat is the figure, all repeats are reported
    rep_ms = []
    for _ in range(max(args.repeats, 1)):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            run()
        e1.record()
        torch.cuda.synchronize()
        rep_ms.append(e0.elapsed_time(e1) / args.steps)
    ms_per_step = sorted(rep_ms)[len(rep_ms) // 2]
    tokens_per_s = wl.tokens / (ms_per_step * 1e-3)
    sclk = sclk_under_load(torch, run) if not args.no_graph else None
    st = step.state()
    loss = float(step.loss)

    # ---- roofline of the dominant kernel, timed live with events on the launch stream: every dense
    # contraction of the step, bracketed where it runs (eager launches of the same step, same buffers)
    step.two_streams = False          # one stream while launches are timed one by one: no other kernel shares the chip
    with GemmTimer(torch, B) as gt:   # untimed pass: creates the event objects (slow the first time in a process;
        step.step()                   # the record of a fresh event would otherwise land late and stretch its bracket)
    del gt
    with GemmTimer(torch, B) as gt:
        for _ in range(args.insitu_steps):
            step.step()
    n_launch, flops, gemm_bytes, raw_secs, empty_secs = gt.totals()
    secs = raw_secs - empty_secs                  # bracket minus empty bracket = the launches themselves
    # the 12 distinct contractions of one layer again, each alone and back to back (operands warm in L2)
    iso_flops, iso_secs, per = gemm_roofline(torch, B, step)
    glue = glue_roofline(torch, B, step, I)
    traffic = traffic_from_summary()
    n_params = step.P.total                       # elements the flat update descriptor covers
    upd_bytes = 28.0 * n_params
    t_upd = _time_calls(torch, lambda: B.mp_unscale_check_update(step.P.flat_list, 1, step.cfg, step.st, 1), 10)
    t_upd_chk = _time_calls(torch, lambda: B.mp_unscale_check_update(step.P.flat_list, 1, step.cfg, step.st, 0), 10)

    # what the matrix cores sustain on this device with register-resident operands: all-zero operands (top clock)
    # and operands distributed like the step's tensors (the clock the chip holds under load depends on the data)
    probe_sink = torch.empty(512 * 256, dtype=torch.float32, device="cuda")
    gen = torch.Generator(device="cuda").manual_seed(1805)
    mfma_rate = {}
    for name, ops in (("zero_operands", torch.zeros(16384, dtype=torch.float16, device="cuda")),
                      ("normal_operands", torch.randn(16384, device="cuda", generator=gen).half())):
        mfma_rate[name] = max(B.mp_mfma_sustained_rate(ops, probe_sink, 512, 60000) for _ in range(2))

    # one plain device copy of known size (256 MiB read + 256 MiB write): the calibration launch for the
    # FETCH_SIZE / WRITE_SIZE counters when this script runs under rocprofv3 --pmc
    cal_src = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()

    out = {
        "metric": "training tokens/sec (fp16 MP step, Transformer-big layer); MFMA util %",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "repeats": len(rep_ms), "ms_per_step_repeats": [round(t, 4) for t in rep_ms],
        "spread_pct": round(100.0 * (max(rep_ms) - min(rep_ms)) / ms_per_step, 2),
        "timing": f"median of {len(rep_ms)} repeats of {args.steps} steps each (HIP events on the stream, no host sync inside)", "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": "config 3: Transformer-big stack, 6 layers, d_model 1024, 16 heads, d_ff 4096, "
                               "64 sequences x 128 tokens = 8192 tokens, fp16 with fp32 masters, MSE, Adam, "
                               "dynamic loss scale 2^15 / growth 100",
                   "launch": "HIP graph replay" if not args.no_graph else "eager ctypes launches",
                   "overflow_check": "in gradient-producing epilogues (MP_UPDATE_PRECHECKED)", "update_list": "one flat descriptor",
                   "streams": "one stream" if args.one_stream else "grouped weight-gradient launch of each layer (with two bias gradients in it) on a second stream"},
        "step_gemm_tflops": wl.gemm_flops_per_step() / (ms_per_step * 1e-3) * 1e-12,
        "step_mfma_util_pct": 100.0 * wl.gemm_flops_per_step() / (ms_per_step * 1e-3) * 1e-12 / PEAK_FP16_TFLOPS,
        "final_loss": loss, "loss_scale": st.scale, "opt_steps": st.opt_step, "skipped": st.skipped_steps,
        "roofline": {"bound": "mfma", "kernel": "gemm_kernel / gemm_dtl_grouped_kernel (every dense fp16 contraction of the step: per layer 4 fwd, 4 dX, and the 4 dW in one grouped launch)",
                     "achieved": flops / secs * 1e-12, "peak": PEAK_FP16_TFLOPS, "unit": "TFLOP/s",
                     "frac": flops / secs * 1e-12 / PEAK_FP16_TFLOPS,
                     "traffic": traffic["gemm"],
                     "launches_timed": n_launch, "launches_per_step": n_launch // max(args.insitu_steps, 1),
                     "avg_launch_us": secs / n_launch * 1e6, "avg_bracket_us": raw_secs / n_launch * 1e6,
                     "avg_empty_bracket_us": empty_secs / n_launch * 1e6, "flops_per_launch": flops / n_launch,
                     "algorithmic_bytes_per_launch": gemm_bytes / n_launch,
                     "isolated": {"achieved": iso_flops / iso_secs * 1e-12, "per_call": per},
                     "sustained_mfma_tflops": mfma_rate,
                     "sclk_mhz_under_load": sclk, "sclk_mhz_max": 2400,
                     "peak_at_sclk_under_load": (PEAK_FP16_TFLOPS * sclk / 2400.0) if sclk else None,
                     "frac_of_peak_at_sclk_under_load": (flops / secs * 1e-12 / (PEAK_FP16_TFLOPS * sclk / 2400.0)) if sclk else None,
                     "frac_of_sustained_normal_operands": flops / secs * 1e-12 / mfma_rate["normal_operands"]},
        "roofline_update": {"bound": "hbm", "kernel": "update_kernel<ADAM> (unscale + Adam + fp16 re-cast)",
                            "achieved": upd_bytes / t_upd * 1e-9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                            "frac": upd_bytes / t_upd * 1e-9 / PEAK_HBM_GBS, "traffic": traffic["update"],
                            "bytes_per_launch": upd_bytes, "us": t_upd * 1e6,
                            "with_inspection_pass_us": t_upd_chk * 1e6,
                            "with_inspection_pass_GBs": (upd_bytes + 2.0 * n_params) / t_upd_chk * 1e-9},
    }
    out["roofline_glue"] = glue
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, I.C2, args.cpu_iterations)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
