#!/usr/bin/env python3
"""Benchmark of the ES-RNN training step on one MI355X.

One step = esrnn_forward + esrnn_backward (every stage of the hot path) over one
batch of synthetic series that is already resident in HBM.  Prints ONE JSON
line: throughput in series-steps/s (one series-step = one time step of one
series; a step processes B*T of them), the roofline position of the dominant
kernel measured with HIP events on the launch stream, and the float64 CPU
oracle timed on the host cores of the same box as a reported baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload quarterly]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3   # MI355X dense fp32 matrix peak
PEAK_HBM_GBS = 8000.0           # MI355X HBM3E peak

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a 256 MiB copy probe
# (FETCH x 2.0, WRITE x 1.0): profiles/hbm_traffic_<workload>_B<batch>.txt.  Valid for that workload and batch only.
MEASURED_TRAFFIC_BYTES = {
    ('tiny_quarterly', 16): {
        "es_forward": 1.1e+05, "window_forward": 1.5e+05, "lstm_forward_l0": 1.05e+06, "lstm_forward_l1": 1.24e+06,
        "lstm_forward_l2": 1.24e+06, "lstm_forward_l3": 1.24e+06, "head_forward_backward": 1.57e+06, "forecasts": 1.4e+05,
        "lstm_backward_l3": 2.54e+06, "lstm_backward_l2": 2.54e+06, "lstm_backward_l1": 2.54e+06, "lstm_backward_l0": 1.33e+06,
        "window_backward": 1.3e+05, "es_backward": 9e+04,
    },
    ('quarterly', 4096): {
        "es_forward": 6.3e+06, "window_forward": 1.421e+07, "lstm_forward_l0": 2.442e+08, "lstm_forward_l1": 3.076e+08,
        "lstm_forward_l2": 3.076e+08, "lstm_forward_l3": 3.076e+08, "head_forward_backward": 1.171e+08, "forecasts": 1.818e+07,
        "lstm_backward_l3": 3.983e+08, "lstm_backward_l2": 3.983e+08, "lstm_backward_l1": 3.983e+08, "lstm_backward_l0": 2.957e+08,
        "window_backward": 1.56e+07, "es_backward": 6.15e+06,
    },
    ('monthly', 4096): {
        "es_forward": 2.019e+07, "window_forward": 1.18e+08, "lstm_forward_l0": 1.121e+09, "lstm_forward_l1": 1.385e+09,
        "lstm_forward_l2": 1.385e+09, "lstm_forward_l3": 1.385e+09, "head_forward_backward": 5.931e+08, "forecasts": 1.317e+08,
        "lstm_backward_l3": 1.697e+09, "lstm_backward_l2": 1.697e+09, "lstm_backward_l1": 1.697e+09, "lstm_backward_l0": 1.355e+09,
        "window_backward": 2.069e+08, "es_backward": 2.005e+07,
    },
    ('yearly', 8192): {
        "es_forward": 5.49e+06, "window_forward": 1.751e+07, "lstm_forward_l0": 1.903e+08, "lstm_forward_l1": 2.341e+08,
        "lstm_forward_l2": 2.341e+08, "lstm_forward_l3": 2.341e+08, "head_forward_backward": 9.038e+07, "forecasts": 1.245e+07,
        "lstm_backward_l3": 2.978e+08, "lstm_backward_l2": 2.978e+08, "lstm_backward_l1": 2.978e+08, "lstm_backward_l0": 2.403e+08,
        "window_backward": 1.543e+07, "es_backward": 4.05e+06,
    },
    ('hourly', 512): {
        "es_forward": 9.58e+06, "window_forward": 9.854e+07, "lstm_forward_l0": 4.217e+08, "lstm_forward_l1": 4.422e+08,
        "lstm_forward_l2": 4.259e+08, "lstm_forward_l3": 4.259e+08, "head_forward_backward": 3.176e+08, "forecasts": 1.318e+08,
        "lstm_backward_l3": 4.99e+08, "lstm_backward_l2": 4.99e+08, "lstm_backward_l1": 5.59e+08, "lstm_backward_l0": 4.417e+08,
        "window_backward": 1.949e+08, "es_backward": 9.44e+06,
    },
}


def stage_model(cfg, name):
    """Algorithmic work of one launch of a stage: (bound, amount, unit).

    Contractions are priced in flops (2 per multiply-add, logical sizes, no
    padding); streaming stages in the bytes the method has to move (fp32)."""
    B, T, I, H, h = cfg.B, cfg.T, cfg.I, cfg.H, cfg.hidden
    P = T - I - H + 1
    n_seas = cfg.n_seas
    if name.startswith("lstm_forward_l") or name.startswith("lstm_backward_l"):
        layer = int(name.rsplit("l", 1)[1])
        k = (I + cfg.n_cat if layer == 0 else h) + h
        per = 2 * k * 4 * h
        if name.startswith("lstm_backward"):
            per *= 2                      # transposed contraction + weight gradient
        return "mfma", float(per) * B * P, "flop"
    if name == "head_forward_backward":
        # bound by its streams: read the top block output and the targets; write outputs, the loss gradient
        # and the gradient of the top block output
        return "hbm", 4.0 * B * P * (2 * h + 3 * H), "byte"
    if name == "forecasts":
        # read outputs, log level and seasonal factors of the target times; write forecasts
        return "hbm", 4.0 * B * P * 2 * H + 4.0 * B * T * (1 + n_seas), "byte"
    if name == "es_forward":
        return "hbm", 4.0 * B * T * (1 + 3 + n_seas) + 4.0 * B * cfg.K, "byte"       # read y; write level, u, v, factors
    if name == "es_backward":
        return "hbm", 4.0 * B * T * (4 + n_seas) + 4.0 * B * cfg.K, "byte"           # read y, level, gu, gv, factors
    if name == "window_forward":
        return "hbm", 4.0 * B * P * (I + H) + 8.0 * B * T, "byte"                     # write X, Z; read u, v
    if name == "window_backward":
        return "hbm", 4.0 * B * P * (I + H) + 8.0 * B * T, "byte"                     # read gX, gO; write gu, gv
    return None, 0.0, ""


def lstm_stash_bytes(cfg, name):
    """Algorithmic HBM bytes of one LSTM layer launch (fp32): the forward pass reads its input and writes the
    activation stash (four activated gates, cell state, hidden state per unit); the reverse pass reads the
    stash, the previous cell and hidden state, the input and the arriving gradient, and writes the input
    gradient.  The last layer of a block >= 1 also reads the block input and writes the block output."""
    B, I, H, h = cfg.B, cfg.I, cfg.H, cfg.hidden
    P = cfg.T - I - H + 1
    layer = int(name.rsplit("l", 1)[1])
    k_in = I + cfg.n_cat if layer == 0 else h
    ends, n = [], 0
    for blk in cfg.blocks:
        n += len(blk)
        ends.append(n - 1)
    residual = layer in ends[1:]
    if name.startswith("lstm_forward"):
        per = k_in + 6 * h + (2 * h if residual else 0)
    else:
        per = 6 * h + 2 * h + k_in + h + k_in
    return 4.0 * per * B * P


def price(cfg, name, ms):
    """Roofline position of one stage: {"ms", bound, achieved, frac, ...}.  An LSTM layer is priced against
    both of its roofs (fp32 MFMA flops and HBM bytes of the stash design) and reported against the tighter one."""
    b, amt, _ = stage_model(cfg, name)
    e = {"ms": round(ms, 4)}
    if b == "mfma":
        tf = amt / (ms * 1e-3) / 1e12
        gbs = lstm_stash_bytes(cfg, name) / (ms * 1e-3) / 1e9
        e.update(tflops=round(tf, 2), frac_mfma_peak=round(tf / PEAK_FP32_MFMA_TFLOPS, 4),
                 gbs=round(gbs, 1), frac_hbm_peak=round(gbs / PEAK_HBM_GBS, 4))
        e["bound"] = "mfma" if e["frac_mfma_peak"] >= e["frac_hbm_peak"] else "hbm"
    elif b == "hbm":
        gbs = amt / (ms * 1e-3) / 1e9
        e.update(gbs=round(gbs, 1), frac_hbm_peak=round(gbs / PEAK_HBM_GBS, 4), bound="hbm")
    return e


def roofline_of(cfg, name, entry):
    """The `roofline` object of the JSON line for the stage `name` priced in `entry`."""
    if entry.get("bound") == "mfma":
        achieved, peak, unit, frac = entry["tflops"], PEAK_FP32_MFMA_TFLOPS, "TFLOP/s", entry["frac_mfma_peak"]
    elif entry.get("bound") == "hbm":
        achieved, peak, unit, frac = entry["gbs"], PEAK_HBM_GBS, "GB/s", entry["frac_hbm_peak"]
    else:
        achieved, peak, unit, frac = 0.0, 1.0, "", 0.0
    out = {"kernel": name, "bound": entry.get("bound"), "achieved": achieved, "peak": peak, "unit": unit, "frac": frac,
           "traffic": MEASURED_TRAFFIC_BYTES.get((cfg.name, cfg.B), {}).get(name),
           "avg_launch_ms": entry["ms"]}
    if "frac_mfma_peak" in entry and "frac_hbm_peak" in entry:
        out["other_bound"] = ({"bound": "hbm", "achieved": entry["gbs"], "unit": "GB/s", "frac": entry["frac_hbm_peak"]}
                              if entry["bound"] == "mfma" else
                              {"bound": "mfma", "achieved": entry["tflops"], "unit": "TFLOP/s", "frac": entry["frac_mfma_peak"]})
    return out


def oracle_baseline(cfg, inp, loss, threads, budget_flops):
    """The float64 CPU oracle as it stands, timed on the host cores on a prefix of the series of the batch
    whose matrix work stays below `budget_flops` (the whole batch if it fits)."""
    from oracle import oracle
    from paper_1907_03329_amd import synth
    if threads > 0:
        oracle.set_num_threads(threads)
    flops = 3.0 * sum(stage_model(cfg, f"lstm_forward_l{l}")[1] for l in range(cfg.n_layers))
    nb = cfg.B
    while nb > 64 and flops * nb / cfg.B > budget_flops:
        nb //= 2
    sub = synth.take_series(inp, range(nb))
    scfg = cfg.with_(B=nb)
    reps = 2

    def oracle_step():
        f = oracle.forward(scfg, sub["y"], sub["lengths"], sub["es_params"], sub["weights"], want_forecasts=True,
                           categories=sub.get("categories"))
        oracle.backward(scfg, f, want_adjoints=False)
        return f

    f = oracle_step()                                  # warm-up, also checks the GPU loss when nb == B
    t1 = time.perf_counter()
    for _ in range(reps):
        oracle_step()
    cpu_s = (time.perf_counter() - t1) / reps
    cpu = {"value": round(nb * cfg.T / cpu_s, 1), "unit": "series-steps/s", "cores": oracle.max_threads(),
           "kind": "oracle",
           "sample": f"{nb} of {cfg.B} series of the same batch, forward+backward, float64, {reps} reps",
           "ms_per_step_sample": round(1e3 * cpu_s, 1)}
    if nb == cfg.B:
        cpu["loss_rel_diff_vs_gpu"] = abs(loss - f.loss) / abs(f.loss)
    return cpu


def measure(cfg, inp, steps, warmup, profile_steps, torch, binding, with_update=False, graph=False):
    """Times `steps` training steps of one workload (inputs already on the device) and the stages of
    `profile_steps` more with the library's HIP events.  Returns a dict of results.  With `graph`, the step is
    also recorded once into a HIP graph (torch's capture on a side stream) and `steps` replays are timed."""
    dev = {k: torch.from_numpy(v).cuda() for k, v in inp.items()}
    step = binding.TrainingStep(cfg, want_forecasts=True)
    if cfg.n_cat:
        step.set_categories(dev["categories"])
    if with_update:
        opt = binding.AdamConfig(1e-4, 1e-4, 0.9, 0.999, 1e-8, 20.0)
        mom = [torch.zeros_like(dev["weights"]), torch.zeros_like(dev["weights"]),
               torch.zeros_like(dev["es_params"]), torch.zeros_like(dev["es_params"])]
        counter = [0]

    def one_step():
        step.forward(dev["y"], dev["lengths"], dev["es_params"], dev["weights"])
        step.backward(dev["y"], dev["lengths"], dev["es_params"], dev["weights"])
        if with_update:
            counter[0] += 1
            binding.esrnn_adam_update(step.handle, opt, counter[0], dev["weights"], step.grad_weights, mom[0], mom[1],
                                      dev["es_params"], step.grad_es_params, mom[2], mom[3], step.workspace)

    for _ in range(warmup):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        one_step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    loss = float(step.loss.item())
    graph_ms = None
    if graph and not with_update:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            one_step()
        for _ in range(warmup):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = round(1e3 * (time.perf_counter() - t0) / steps, 4)
        assert abs(float(step.loss.item()) - loss) <= 1e-6 * abs(loss), "the replayed step gives another loss"
        del g
    # per-stage durations: HIP events recorded by the library on the launch stream
    binding.esrnn_profile_enable(step.handle, True)
    for _ in range(max(1, profile_steps)):
        one_step()
        binding.esrnn_profile_collect(step.handle)
    stages = binding.esrnn_profile_read(step.handle)
    binding.esrnn_profile_enable(step.handle, False)
    stage_ms = {name: tot / max(cnt, 1) for name, tot, cnt in stages if cnt}
    report = {name: price(cfg, name, ms) for name, ms in stage_ms.items()}
    dominant = max(stage_ms, key=stage_ms.get)
    step.close()
    del step, dev
    per_step = elapsed / steps
    return {"ms_per_step": round(1e3 * per_step, 4), "value": round(cfg.B * cfg.T / per_step, 1),
            "ms_per_step_graph_replay": graph_ms,
            "window_steps_per_s": round(cfg.B * cfg.P / per_step, 1), "loss": loss, "stages": report,
            "sum_stage_ms": round(sum(stage_ms.values()), 4), "roofline": roofline_of(cfg, dominant, report[dominant])}


def epoch_benchmark(args, cfg, torch, binding, synth):
    """One epoch over a store of N series in random batches of B: esrnn_gather_batch, esrnn_forward,
    esrnn_backward, esrnn_adam_update_indexed per batch (a last partial batch is dropped).  The paper trains
    15 epochs on at most 24000 quarterly series (Tables 2 and 5); its 8.94 min are context, other hardware."""
    import numpy as np
    N = args.epoch
    store = synth.make_inputs(cfg.with_(B=N), seed=0, ragged=True)
    d = {k: torch.from_numpy(v).cuda() for k, v in store.items()}
    step = binding.TrainingStep(cfg, want_forecasts=False)
    opt = binding.AdamConfig(1e-4, 1e-4, 0.9, 0.999, 1e-8, 20.0)
    w = d["weights"]
    m_w, v_w = torch.zeros_like(w), torch.zeros_like(w)
    m_e, v_e = torch.zeros_like(d["es_params"]), torch.zeros_like(d["es_params"])
    counts = torch.zeros(N, dtype=torch.int32, device="cuda")
    y = torch.empty((cfg.T, cfg.B), dtype=torch.float32, device="cuda")
    n = torch.empty(cfg.B, dtype=torch.int32, device="cuda")
    es = torch.empty((cfg.K, cfg.B), dtype=torch.float32, device="cuda")
    nb = N // cfg.B
    rng = np.random.default_rng(0)
    t = [0]

    def epoch():
        perm = torch.from_numpy(rng.permutation(N).astype(np.int32)).cuda()
        for s in range(nb):
            idx = perm[s * cfg.B:(s + 1) * cfg.B]
            t[0] += 1
            binding.esrnn_gather_batch(step.handle, d["y"], d["lengths"], d["es_params"], idx, y, n, es)
            step.forward(y, n, es, w)
            step.backward(y, n, es, w)
            binding.esrnn_adam_update_indexed(step.handle, opt, t[0], w, step.grad_weights, m_w, v_w, d["es_params"],
                                              step.grad_es_params, m_e, v_e, counts, idx, step.workspace)

    epoch()                                   # warm-up epoch
    torch.cuda.synchronize()
    loss0 = float(step.loss.item())
    reps = 3
    t0 = time.perf_counter()
    for _ in range(reps):
        epoch()
    torch.cuda.synchronize()
    el = (time.perf_counter() - t0) / reps
    series_steps = float(store["lengths"][:nb * cfg.B].sum())      # valid time steps; ragged lengths
    print(json.dumps({"metric": "training series-steps/sec over an epoch (gather + fwd + bwd + indexed Adam)",
                      "value": round(nb * cfg.B * cfg.T / el, 1), "unit": "series-steps/s", "n_gpus": 1,
                      "ms_per_epoch": round(1e3 * el, 3), "batches_per_epoch": nb, "ms_per_batch": round(1e3 * el / nb, 4),
                      "higher_is_better": True, "dtype": "f32", "data": "synthetic, ragged lengths",
                      "config": {"workload": cfg.name, "N": N, "B": cfg.B, "T": cfg.T},
                      "unpadded_series_steps_per_s": round(series_steps / el, 1),
                      "loss_after_first_epoch": loss0, "loss_after_last_epoch": float(step.loss.item()),
                      "epochs_timed": reps}))
    step.close()


def es_window_sweep(args, torch, binding, synth):
    """Smoothing and window stages alone at large batch sizes (their HBM roofline is only meaningful there:
    at the benchmark batch a 72-step dependent chain on 64 waves is latency-bound)."""
    import ctypes
    for B in [int(x) for x in args.es_window_sweep.split(",")]:
        cfg = synth.CONFIGS[args.workload].with_(B=B)
        inp = synth.make_inputs(cfg, seed=0)
        dev = {k: torch.from_numpy(v).cuda() for k, v in inp.items() if k != "weights"}
        h = binding.esrnn_create(cfg)
        nbytes = binding.esrnn_es_window_workspace_bytes(h)
        ws = torch.zeros(nbytes // 4, dtype=torch.float32, device="cuda")
        ges = torch.empty((cfg.K, B), dtype=torch.float32, device="cuda")

        def one():
            binding.esrnn_es_window_forward(h, dev["y"], dev["lengths"], dev["es_params"], ws)
            binding.esrnn_es_window_backward(h, dev["y"], dev["lengths"], dev["es_params"], ws, ges)

        for _ in range(3):
            one()
        torch.cuda.synchronize()
        binding.esrnn_profile_enable(h, True)
        for _ in range(max(1, args.profile_steps)):
            one()
            binding.esrnn_profile_collect(h)
        stages = {n: t / max(c, 1) for n, t, c in binding.esrnn_profile_read(h) if c}
        binding.esrnn_profile_enable(h, False)
        out = {"workload": cfg.name, "B": B, "T": cfg.T, "workspace_MB": round(nbytes / 1e6, 1), "stages": {}}
        for name, ms in stages.items():
            bound, amt, _ = stage_model(cfg, name)
            e = {"ms": round(ms, 4)}
            if bound == "hbm":
                e["gbs"] = round(amt / (ms * 1e-3) / 1e9, 1)
                e["frac_hbm_peak"] = round(e["gbs"] / PEAK_HBM_GBS, 4)
            out["stages"][name] = e
        print(json.dumps(out), flush=True)
        binding.esrnn_destroy(h)
        del ws, ges, dev


def config_summary(cfg, with_update=False):
    return {"workload": cfg.name, "B": cfg.B, "T": cfg.T, "seasons": [m for m in (cfg.m1, cfg.m2) if m],
            "I": cfg.I, "H": cfg.H, "hidden": cfg.hidden, "dilations": [list(b) for b in cfg.blocks],
            "tau": cfg.tau, "lambda_lv": cfg.lambda_lv, "window_steps": cfg.B * cfg.P,
            "parameter_update": bool(with_update), "categories": cfg.n_cat}


def issue_overlap_probe(torch, binding, iterations=2000):
    """Times the four modes of esrnn_probe_issue_overlap with one and two workgroups per compute unit."""
    torch.cuda.set_device(0)
    out = torch.empty(2 * 256 * 256, dtype=torch.float32, device="cuda")
    names = {0: "mfma_only", 1: "vector_fma_only", 2: "both_in_every_wave", 3: "mfma_workgroup_beside_fma_workgroup"}
    res = {}
    for per_cu in (1, 2):
        for mode in (0, 1, 2, 3):
            if mode == 3 and per_cu == 1:
                continue
            best = None
            for _ in range(3):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                binding.esrnn_probe_issue_overlap(mode, iterations, per_cu, out)
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1)
                best = ms if best is None else min(best, ms)
            res[f"{names[mode]}_{per_cu}_per_cu"] = round(best * 1e6 / iterations, 1)
    print(json.dumps({"probe": "issue overlap of fp32 MFMA (16x16x4) and vector FMA on one SIMD",
                      "unit": "ns per round of 16 MFMAs and/or 64 vector FMAs per wave",
                      "iterations": iterations, "workgroups": "256 x per_cu, four waves each", **res}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="quarterly",
                    help="the headline workload is quarterly (B=4096); with the default, the JSON line also carries "
                         "the other four workloads under \"workloads\" unless --only-headline is given")
    ap.add_argument("--only-headline", action="store_true", help="time the named workload only")
    ap.add_argument("--batch", type=int, default=0, help="override the number of series")
    ap.add_argument("--profile-steps", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-threads", type=int, default=0, help="host threads of the oracle baseline (0 = all)")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run one device-to-device copy of this many MiB (reference for scaling rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--categories", type=int, default=0,
                    help="feed a one-hot block of this many series categories after the input window (the paper "
                         "uses 6); 0 = the headline configuration")
    ap.add_argument("--with-update", action="store_true",
                    help="add the clipped Adam update (esrnn_adam_update) to every step: the training loop rather "
                         "than the headline forward+backward step")
    ap.add_argument("--graph", action="store_true",
                    help="also record the step once into a HIP graph and time its replays (ms_per_step_graph_replay); "
                         "the headline value stays the eager one")
    ap.add_argument("--predict", action="store_true",
                    help="time esrnn_predict (out-of-sample forecasts of every series, lengths T - H) instead of "
                         "the training step; one JSON line, not the headline metric")
    ap.add_argument("--ragged", default="", choices=["", "sorted", "unsorted"],
                    help="draw ragged lengths (the fraction 652/912 .. 1 of T, the range of lengths of the paper's hourly "
                         "series, Table 3) and time the training step with the series sorted by length or in random "
                         "order; the JSON line also carries the full-length time of the same batch")
    ap.add_argument("--epoch", type=int, default=0,
                    help="train one epoch over a store of this many synthetic series of the workload's shape (the paper's "
                         "quarterly set has 24000, Table 2) in batches of B: gather, forward, backward, indexed Adam "
                         "update per batch; reports series-steps/s over the epoch instead of the headline line")
    ap.add_argument("--es-window-sweep", default="",
                    help="comma-separated batch sizes: time only the smoothing and window stages (forward and "
                         "adjoint) at each, one JSON line per size, instead of the training-step benchmark")
    ap.add_argument("--issue-overlap-probe", action="store_true",
                    help="time the library's synthetic probe kernel (fp32 MFMAs, vector FMAs, both) and print one "
                         "JSON line: do the two kinds of instruction overlap on a SIMD? (not a benchmark of the method)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (series shard trivially across GPUs, "
              "but no multi-GPU path is built); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1907_03329_amd import binding, synth

    if args.es_window_sweep:
        es_window_sweep(args, torch, binding, synth)
        return
    if args.issue_overlap_probe:
        issue_overlap_probe(torch, binding)
        return
    cfg = synth.CONFIGS[args.workload]
    if args.batch:
        cfg = cfg.with_(B=args.batch)
    if args.categories:
        cfg = cfg.with_(n_cat=args.categories)
    inp = synth.make_inputs(cfg, seed=0)
    torch.cuda.set_device(0)

    if args.copy_probe_mib:
        src = torch.ones(args.copy_probe_mib * 262144, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.epoch:
        epoch_benchmark(args, cfg, torch, binding, synth)
        return

    if args.ragged:
        import numpy as np
        full = measure(cfg, inp, args.steps, args.warmup, args.profile_steps, torch, binding)
        rng = np.random.default_rng(1)
        lo = max(int(np.ceil(cfg.T * 652.0 / 912.0)), cfg.I + cfg.H + max(cfg.m1, cfg.m2, 2))
        n = rng.integers(lo, cfg.T + 1, size=cfg.B).astype(np.int32)
        if args.ragged == "sorted":
            n = np.sort(n)[::-1].copy()
        rinp = dict(inp)
        rinp["lengths"] = n
        rinp["y"] = inp["y"].copy()
        rinp["y"][np.arange(cfg.T)[:, None] >= n[None, :]] = 1.0
        m = measure(cfg, rinp, args.steps, args.warmup, args.profile_steps, torch, binding)
        frac = float(n.sum()) / (cfg.B * cfg.T)
        print(json.dumps({"metric": "training-step series-steps/sec (fwd+bwd), ragged batch", "order": args.ragged,
                          "value": round(float(n.sum()) / (m["ms_per_step"] * 1e-3), 1), "unit": "unpadded series-steps/s",
                          "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": m["ms_per_step"],
                          "ms_per_step_full_length": full["ms_per_step"], "filled_fraction": round(frac, 4),
                          "time_fraction": round(m["ms_per_step"] / full["ms_per_step"], 4),
                          "higher_is_better": True, "dtype": "f32", "data": "synthetic",
                          "config": config_summary(cfg), "stages": m["stages"]}))
        return

    if args.predict:
        import numpy as np
        dev = {k: torch.from_numpy(v).cuda() for k, v in inp.items()}
        step = binding.TrainingStep(cfg, want_forecasts=True)
        if args.categories:
            step.set_categories(dev["categories"])
        n = torch.from_numpy(np.full(cfg.B, cfg.T - cfg.H, dtype=np.int32)).cuda()
        for _ in range(args.warmup):
            out = step.predict(dev["y"], n, dev["es_params"], dev["weights"])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            out = step.predict(dev["y"], n, dev["es_params"], dev["weights"])
        torch.cuda.synchronize()
        el = (time.perf_counter() - t0) / args.steps
        binding.esrnn_profile_enable(step.handle, True)
        for _ in range(max(1, args.profile_steps)):
            step.predict(dev["y"], n, dev["es_params"], dev["weights"])
            binding.esrnn_profile_collect(step.handle)
        stages = {name: round(tot / max(cnt, 1), 4) for name, tot, cnt in binding.esrnn_profile_read(step.handle) if cnt}
        print(json.dumps({"metric": "out-of-sample forecast series/sec (H steps each)", "value": round(cfg.B / el, 1),
                          "unit": "series/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                          "ms_per_step": round(1e3 * el, 4), "higher_is_better": True, "dtype": "f32",
                          "data": "synthetic", "config": {"workload": cfg.name, "B": cfg.B, "T": cfg.T, "H": cfg.H},
                          "series_steps_per_s": round(cfg.B * (cfg.T - cfg.H) / el, 1), "stages_ms": stages,
                          "mean_forecast": float(out.mean().item())}))
        return

    m = measure(cfg, inp, args.steps, args.warmup, args.profile_steps, torch, binding, with_update=args.with_update,
                graph=args.graph)
    cpu = None
    if not args.no_cpu_baseline:
        cpu = oracle_baseline(cfg, inp, m["loss"], args.cpu_threads, 1.2e11)

    # The other workloads, when the default headline run is asked for: same measurement, fewer steps, a
    # smaller sample for the oracle, so that the whole run stays within a few minutes.
    others = None
    plain = (args.workload == "quarterly" and not args.batch and not args.categories and not args.with_update
             and not args.only_headline)
    if plain:
        others = {}
        for name in synth.CONFIG_ORDER:
            if name == cfg.name:
                continue
            ocfg = synth.CONFIGS[name]
            oinp = synth.make_inputs(ocfg, seed=0)
            om = measure(ocfg, oinp, max(10, args.steps // 4), max(3, args.warmup // 2), max(3, args.profile_steps // 4),
                         torch, binding)
            entry = {"config": config_summary(ocfg), "ms_per_step": om["ms_per_step"], "value": om["value"],
                     "unit": "series-steps/s", "window_steps_per_s": om["window_steps_per_s"], "loss": om["loss"],
                     "roofline": om["roofline"], "stages": om["stages"], "sum_stage_ms": om["sum_stage_ms"]}
            if not args.no_cpu_baseline:
                entry["cpu_baseline"] = oracle_baseline(ocfg, oinp, om["loss"], args.cpu_threads, 3e10)
            others[name] = entry

    out = {
        "metric": "training-step series-steps/sec (fwd+bwd)",
        "value": m["value"],
        "unit": "series-steps/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": m["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": config_summary(cfg, args.with_update),
        "window_steps_per_s": m["window_steps_per_s"],
        "loss": m["loss"],
        "roofline": m["roofline"],
        "cpu_baseline": cpu,
        "stages": m["stages"],
        "sum_stage_ms": m["sum_stage_ms"],
    }
    if m["ms_per_step_graph_replay"] is not None:
        out["ms_per_step_graph_replay"] = m["ms_per_step_graph_replay"]
    if others is not None:
        out["workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
