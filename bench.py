#!/usr/bin/env python3
"""Benchmark of the uniformly-sparse output layer's train step on one MI355X.

One step = forward + sparse-target BCE (loss and gradient) + backward-weight + backward-input +
Adam, plus a connection redistribution after every `period`-th step, on seeded synthetic data
of the headline workload (m=500,000 labels, d=32,768, fan-in k=32, batch 256, float32).
All inputs are resident in HBM before the timed region starts.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published peak

# HBM-side bytes per call measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by what the
# same counters read for a plain copy of known size); summary and commands in
# profiles/train_step_large_f32_hbm_bytes.txt.  Only the workload it was measured on has an entry.
MEASURED_TRAFFIC_BYTES = {
    "large": {"backward_input": 5527399 * 1024, "forward": 903295 * 1024, "backward_weight": 918642 * 1024},
}
KERNELS_OF_CALL = {
    "forward": "k_forward (1 launch)",
    "bce": "k_bce + k_bce_finish",
    "backward_weight": "k_backward_weight (1 launch)",
    "backward_input": "k_gather_w + k_transpose_g + one k_bwd_input_window per label window + k_untile",
    "adam": "k_adam (1 launch)",
}


def algorithmic_bytes(cfg):
    """Bytes each call has to move at the C-ABI level (x counted once per pass)."""
    es = 2 if cfg.storage == "bf16" else 4
    E, N, X = cfg.b * cfg.m, cfg.m * cfg.k, cfg.b * cfg.d
    per = {
        "forward": (4 + es) * N + es * X + 4 * E,
        "bce": 8 * E,
        "backward_weight": 4 * E + 4 * N + es * X + 4 * N,
        "backward_input": 4 * E + (4 + es) * N + 4 * X,
        "adam": (es + 12) * N + (es + 8) * N,
    }
    per["step"] = sum(per.values())
    return per


def cpu_baseline(cfg, budget_s=12.0, max_reps=5):
    """The oracle, as it stands, timed on the host cores on the same workload: whole train steps
    (forward, BCE, backward-weight, backward-input, Adam) of one full batch, repeated until about
    `budget_s` seconds of CPU work have been spent."""
    import oracle
    import workloads as wl
    idx, W, x = wl.gen_idx(cfg), wl.gen_W(cfg), wl.gen_x(cfg)
    off, lab = wl.gen_targets(cfg)
    m1 = np.zeros((cfg.m, cfg.k), np.float32)
    m2 = np.zeros((cfg.m, cfg.k), np.float32)
    hp = wl.ADAM
    times = []
    while len(times) < max_reps and (not times or sum(times) < budget_s):
        t0 = time.perf_counter()
        out = oracle.forward(x, idx, W)
        _, g = oracle.bce_loss_grad(out, off, lab, 1.0 / cfg.b)
        gW = oracle.backward_weight(g, x, idx)
        oracle.backward_input(g, idx, W, cfg.d)
        oracle.adam_step(W, gW, m1, m2, len(times) + 1, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"])
        times.append(time.perf_counter() - t0)
    per_step = float(np.mean(times))
    return {"value": 1.0 / per_step, "unit": "steps/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%d whole train steps (no redistribution) of the same workload, full batch of %d; "
                      "%.2f s per step" % (len(times), cfg.b, per_step)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="large", help="tiny | medium | large | large_wide | stress")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for scaling rocprofv3 byte counters)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the squared-hinge sweep and the prediction timing that a default run at N=1 appends")
    ap.add_argument("--sqh-sweep", action="store_true",
                    help="also time the squared-hinge loss and the two backward calls on gradients with "
                         "0 / 90 / 99 / 99.9 %% exact zeros (implicit negative mining, Section 3.3)")
    ap.add_argument("--separate-calls", action="store_true",
                    help="time the step as five separate calls instead of usl_train_step")
    ap.add_argument("--predict", action="store_true",
                    help="also time prediction (Section 2): top-5 labels of every score row and the P@k hit counts")
    ap.add_argument("--traffic-kib", type=float, default=None,
                    help="HBM KiB per launch of the dominant kernel from rocprofv3 --pmc (FETCH+WRITE, scaled)")
    args = ap.parse_args()
    if not args.no_extras and not args.no_cpu_baseline and args.workload == "large":
        args.sqh_sweep = args.predict = True     # the default run also reports the widened rows
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as wl
    from paper_2306_03725_amd import usl   # raises if libusl.so is not built: no fallback

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    cfg = wl.CONFIGS[args.workload]
    m, d, k, b = cfg.m, cfg.d, cfg.k, cfg.b
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()
    L = usl.Layer(m, d, k, b, cfg.storage, stream.cuda_stream)

    def up(a):
        a = np.ascontiguousarray(a)
        if a.dtype == np.uint16:
            a = a.view(np.int16)
        return torch.from_numpy(a).to(dev)

    # ---- resident state and inputs
    idx = torch.empty((m, k), dtype=torch.int32, device=dev)
    L.init_indices(idx, 1000 * cfg.index + wl.STREAM_IDX)
    W = up(wl.gen_W(cfg))
    m1 = torch.zeros((m, k), dtype=torch.float32, device=dev)
    m2 = torch.zeros((m, k), dtype=torch.float32, device=dev)
    gW = torch.empty((m, k), dtype=torch.float32, device=dev)
    xs = [up(wl.gen_x(cfg, i)) for i in range(cfg.n_x_batches)]
    tg = [tuple(up(a) for a in wl.gen_targets(cfg, i)) for i in range(cfg.n_x_batches)]
    out = torch.empty((b, m), dtype=torch.float32, device=dev)     # g is written in place
    gx = torch.empty((b, d), dtype=torch.float32, device=dev)
    loss = torch.empty((1,), dtype=torch.float32, device=dev)
    seed = wl.redistribution_seed(cfg)
    scale = float(np.float32(1.0 / b))
    hp = wl.ADAM
    state = {"t": 0, "epoch": 0}
    calls = ["forward", "bce", "backward_weight", "backward_input", "adam", "redistribute"]

    def step(ev=None):
        state["t"] += 1
        t = state["t"]
        x = xs[t % len(xs)]
        off, lab = tg[t % len(tg)]
        marks = []

        def mark():
            if ev is not None:
                e = torch.cuda.Event(enable_timing=True)
                e.record(stream)
                marks.append(e)
        mark()
        L.forward(x, idx, W, out, b); mark()
        L.bce_loss_grad(out, off, lab, scale, out, loss, b); mark()
        L.backward_weight(out, x, idx, gW, b); mark()
        L.backward_input(out, idx, W, gx, b); mark()
        L.adam_step(W, gW, m1, m2, t, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"]); mark()
        if wl.is_redistribution_step(cfg, t):
            L.redistribute(idx, W, m1, m2, cfg.fraction, seed, state["epoch"])
            state["epoch"] += 1
            mark()
        if ev is not None:
            ev.append(marks)

    def fused_step():
        state["t"] += 1
        t = state["t"]
        x = xs[t % len(xs)]
        off, lab = tg[t % len(tg)]
        L.train_step(x, idx, W, m1, m2, off, lab, 0, scale, t, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"],
                     out, gW, gx, loss, b)
        if wl.is_redistribution_step(cfg, t):
            L.redistribute(idx, W, m1, m2, cfg.fraction, seed, state["epoch"])
            state["epoch"] += 1

    timed_step = step if args.separate_calls else fused_step
    for _ in range(args.warmup):
        timed_step()
    torch.cuda.synchronize()
    if args.calibrate_copy:    # 2^30 bytes read + 2^30 bytes written by one elementwise kernel
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    # ---- the timed region: exactly args.steps steps
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_wall0 = time.perf_counter()
    e0.record(stream)
    for _ in range(args.steps):
        timed_step()
    e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_wall0) * 1e3
    total_ms = e0.elapsed_time(e1)
    loss_value = float(loss.item())
    # ---- the same steps as separate calls with an event between the calls: the per-call breakdown
    events = []
    step()
    s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s0.record(stream)
    for _ in range(args.steps):
        step(events)
    s1.record(stream)
    torch.cuda.synchronize()
    separate_ms = s0.elapsed_time(s1) / args.steps
    n_bad = L.validate_indices(idx)

    per_call = {c: [] for c in calls}
    for marks in events:
        for i in range(len(marks) - 1):
            per_call[calls[i]].append(marks[i].elapsed_time(marks[i + 1]))
    call_ms = {c: (float(np.mean(v)) if v else None) for c, v in per_call.items()}
    ab = algorithmic_bytes(cfg)
    ms_per_step = total_ms / args.steps
    steps_per_s = 1e3 / ms_per_step
    # the dominant call and its roofline position (algorithmic bytes / measured time)
    dom = max((c for c in calls[:5]), key=lambda c: call_ms[c] or 0.0)
    dom_gbps = ab[dom] / (call_ms[dom] * 1e-3) / 1e9
    traffic = MEASURED_TRAFFIC_BYTES.get(cfg.name, {}).get(dom)
    if args.traffic_kib is not None:
        traffic = args.traffic_kib * 1024
    roof = {"bound": "hbm", "kernel": "usl_%s: %s" % (dom, KERNELS_OF_CALL[dom]),
            "achieved": round(dom_gbps, 1), "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": round(dom_gbps / HBM_PEAK_GBPS, 4),
            "ms_per_launch": round(call_ms[dom], 4), "algorithmic_bytes": ab[dom],
            "traffic": traffic,
            "note": "dominant call of the step; achieved = algorithmic bytes / HIP-event time of the call; "
                    "traffic = HBM bytes per call from rocprofv3 counters (profiles/), measured offline"}
    step_gbps = ab["step"] / (ms_per_step * 1e-3) / 1e9
    res = {
        "metric": "sparse_layer_train_steps_per_s", "value": round(steps_per_s, 2), "unit": "steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if cfg.storage == "f32" else "bf16 storage, f32 arithmetic", "data": "synthetic",
        "config": {"workload": "%s: m=%d d=%d k=%d b=%d %s, redistribution of %.0f%% every %d steps"
                               % (cfg.name, m, d, k, b, cfg.storage, 100 * cfg.fraction, cfg.period),
                   "parallelism": "single GPU"},
        "achieved_hbm_GBps": round(step_gbps, 1), "hbm_frac_of_peak": round(step_gbps / HBM_PEAK_GBPS, 4),
        "algorithmic_GB_per_step": round(ab["step"] / 1e9, 4),
        "call_ms": {c: (round(v, 4) if v is not None else None) for c, v in call_ms.items()},
        "call_GBps": {c: round(ab[c] / (call_ms[c] * 1e-3) / 1e9, 1) for c in calls[:5]},
        "wall_ms_per_step": round(wall_ms / args.steps, 4),
        "timed_path": ("separate calls: usl_forward, usl_bce_loss_grad, usl_backward_weight, usl_backward_input, "
                       "usl_adam_step" if args.separate_calls else "usl_train_step (the same five stages in one call)")
                      + ", usl_redistribute on its schedule",
        "separate_calls_ms_per_step": round(separate_ms, 4),
        "loss": loss_value, "bad_rows": n_bad, "redistributions": state["epoch"],
        "roofline": roof,
    }
    if args.sqh_sweep:
        try:
            # Synthetic stand-in for the gradient of a trained model under the squared hinge loss: the
            # scores' own gradient with a seeded share of entries forced to exactly zero.
            def timed(fn, reps=5):
                fn()
                a, z = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record(stream)
                for _ in range(reps):
                    fn()
                z.record(stream)
                torch.cuda.synchronize()
                return a.elapsed_time(z) / reps
            x0 = xs[0]
            off0, lab0 = tg[0]
            L.forward(x0, idx, W, out, b)
            sweep = {}
            gbuf = torch.empty_like(out)
            sweep["sqh_loss_ms"] = round(timed(lambda: L.sqh_loss_grad(out, off0, lab0, scale, gbuf, loss, b)), 4)
            gen = torch.Generator(device=dev)
            gen.manual_seed(1000 * cfg.index + 77)
            for frac in (0.0, 0.9, 0.99, 0.999):
                L.sqh_loss_grad(out, off0, lab0, scale, gbuf, loss, b)
                if frac > 0:
                    keep = torch.rand(gbuf.shape, generator=gen, device=dev) >= frac
                    gbuf.mul_(keep)
                    del keep
                nz = float((gbuf != 0).float().mean().item())
                sweep["zero_frac_%g" % frac] = {
                    "nonzero_share": round(nz, 5),
                    "backward_weight_ms": round(timed(lambda: L.backward_weight(gbuf, x0, idx, gW, b)), 4),
                    "backward_input_ms": round(timed(lambda: L.backward_input(gbuf, idx, W, gx, b)), 4)}
            res["sqh_zero_skipping"] = sweep
            del gbuf
        except Exception as exc:   # the headline line must survive a failure of an appended leg
            res['sqh_zero_skipping'] = {"error": repr(exc)}
    if args.predict:
        try:
            kk = 5
            L.forward(xs[0], idx, W, out, b)
            top_lab = torch.empty((b, kk), dtype=torch.int32, device=dev)
            top_val = torch.empty((b, kk), dtype=torch.float32, device=dev)
            hits = torch.empty((kk,), dtype=torch.int64, device=dev)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            reps = 10
            L.topk(out, b, kk, top_lab, top_val)
            ev[0].record(stream)
            for _ in range(reps):
                L.topk(out, b, kk, top_lab, top_val)
            ev[1].record(stream)
            for _ in range(reps):
                L.precision_hits(top_lab, tg[0][0], tg[0][1], b, kk, hits)
            ev[2].record(stream)
            torch.cuda.synchronize()
            t_top = ev[0].elapsed_time(ev[1]) / reps
            pe = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            L.predict(xs[0], idx, W, b, kk, top_lab, top_val)
            pe[0].record(stream)
            for _ in range(reps):
                L.predict(xs[0], idx, W, b, kk, top_lab, top_val)
            pe[1].record(stream)
            torch.cuda.synchronize()
            res["predict"] = {"kk": kk, "predict_ms": round(pe[0].elapsed_time(pe[1]) / reps, 4), "topk_ms": round(t_top, 4),
                              "topk_GBps": round(4.0 * b * m / (t_top * 1e-3) / 1e9, 1),
                              "precision_hits_ms": round(ev[1].elapsed_time(ev[2]) / reps, 4),
                              "hits": hits.tolist()}
        except Exception as exc:   # the headline line must survive a failure of an appended leg
            res['predict'] = {"error": repr(exc)}
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
