#!/usr/bin/env python3
"""Benchmark of the uniformly-sparse output layer's train step on one MI355X.

One step = forward + sparse-target BCE (loss and gradient) + the two backward products (weight and input
gradient) + Adam, plus a connection redistribution after every `period`-th step, on seeded synthetic data
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

# HBM-side bytes per call measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (each scaled by what the same
# counter reads for a plain copy of known size); summaries and commands in profiles/train_step_<workload>_*_hbm_bytes.txt.
# They are measured offline (a counter run serialises the kernels) and go stale when a kernel changes: the
# profile files carry the date of truth, these constants only repeat their per-call totals.
MEASURED_TRAFFIC_BYTES = {
    "large": {"backward": 3903848448, "backward_input": 2844157542, "forward": 924948889, "backward_weight": 940782387},
    "large_wide": {"backward": 17392939827, "backward_input": 8593394892, "forward": 2478204518, "backward_weight": 2651114700},
    "stress": {"backward": 178784619724, "backward_input": 203820315443, "forward": 26037190656, "backward_weight": 26132296499},
}
KERNELS_OF_CALL = {
    "forward": "k_forward (1 launch)",
    "bce": "k_bce + k_bce_finish",
    "backward_weight": "k_backward_weight (1 launch)",
    "backward_input": "a look at a sample of g, k_gather_w, then per group of 256 instances k_transpose_g + one "
                      "k_bwd_input_window per window of 24576 labels + k_untile",
    "backward_input_register_lists": "a look at a sample of g, k_idx_fingerprint, then per pass over the batch "
                                     "k_bwi_lds (lists in registers, rows of g through LDS) + k_lf_reduce",
    "backward": "usl_backward_weight's and usl_backward_input's kernels, one call after the other",
    "backward_one_pass": "a look at a sample of g, k_idx_fingerprint, k_both_lds (both products from one pass over g: "
                         "lists in registers with a weight-gradient sum per connection, two rows of g through LDS at a "
                         "time) + k_lf_reduce + k_unstage (the weight gradient into slot order)",
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
    # usl_backward is scored against the bytes of the two separate calls it stands for; read once, g, idx and the
    # list of connections would be 4E + (8 + es)N + (es + 4)X
    per["backward"] = per["backward_weight"] + per["backward_input"]
    per["backward_one_pass_lower_bound"] = 4 * E + (8 + es) * N + (es + 4) * X
    return per


PARTIAL_SUM_BYTES = 16 << 30   # what the library lets the partial sums of a pass over the batch take on this device


def register_list_windows(cfg, cus=256):
    """Label windows of usl_backward_input's register-list form for this shape, or 0 where the library keeps the other
    form (its rule: windows of 16384 to 32768 labels that send about 32 connections into a feature, whole blocks of
    2048 features, enough workgroups to fill the chip; the windows shortened until the rounds of workgroups are full)."""
    lists32 = 32 * cfg.d // cfg.k
    if not (cfg.d % 2048 == 0 and cfg.d <= 65536 and cfg.m % 4 == 0 and 16384 <= lists32 <= 32768):
        return 0
    cap = min(lists32, 32768) // 4 * 4
    nwin, nfb = -(-cfg.m // cap), cfg.d // 2048
    if nwin * nfb * 4 < cus * 3:
        return 0
    full = -(-nwin * nfb // cus) * cus // nfb
    return full if nwin < full <= nwin * 5 // 4 else nwin


def register_list_form(cfg):
    return register_list_windows(cfg) > 0


def one_pass_windows(cfg, cus=256):
    """Label windows of usl_backward's one-pass form (both products from one pass over g), or 0 where the library runs
    the two separate products (its rule: windows of 8192 to 15968 labels that send 16 connections or fewer into a
    feature, whole blocks of 2048 features, enough workgroups to fill the chip)."""
    lists16 = 16 * cfg.d // cfg.k
    if not (cfg.d % 2048 == 0 and cfg.d <= 65536 and cfg.m % 4 == 0 and 8192 <= lists16 <= 32768):
        return 0
    cap = min(lists16, 15968) // 4 * 4
    nwin, nfb = -(-cfg.m // cap), cfg.d // 2048
    full = -(-nwin * nfb // cus) * cus // nfb
    nwin = full if nwin < full <= nwin * 5 // 4 else nwin
    if nwin * nfb * 4 < cus * 3 or nwin * 64 * cfg.d * 4 > PARTIAL_SUM_BYTES:
        return 0
    return nwin


def launches_in_call(cfg, call):
    """Kernel launches behind one call (the HIP-event time of the call covers all of them)."""
    if call == "backward":
        nwin = one_pass_windows(cfg)
        if nwin:
            rows = max(64, min(cfg.b, PARTIAL_SUM_BYTES // (nwin * cfg.d * 4))) & ~1
            return 3 + 2 * -(-cfg.b // rows) + 1
        return launches_in_call(cfg, "backward_weight") + launches_in_call(cfg, "backward_input")
    if call != "backward_input":
        return 2 if call == "bce" else 1
    groups = -(-cfg.b // 256)
    nwin = register_list_windows(cfg)
    if nwin:
        passes = -(-cfg.b // max(64, min(cfg.b, PARTIAL_SUM_BYTES // (nwin * cfg.d * 4))))
        return 3 + passes * 2
    win = int((24576.0 * ((cfg.d / 32768.0) * (32.0 / cfg.k)) ** 0.5 + 2048.0) / 4096.0) * 4096   # labels per window,
    win = min(max(win, 16384), 49152)                                                              # as the library picks them
    return 3 + groups * (1 + -(-cfg.m // win) + 1 + 1)


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


class Bench:
    """Resident state and inputs of one workload, and the two ways of running a step."""

    def __init__(self, cfg, torch, usl, wl):
        self.cfg, self.torch, self.wl = cfg, torch, wl
        m, d, k, b = cfg.m, cfg.d, cfg.k, cfg.b
        dev = torch.device("cuda:0")
        self.stream = torch.cuda.current_stream()
        self.L = usl.Layer(m, d, k, b, cfg.storage, self.stream.cuda_stream)

        def up(a):
            a = np.ascontiguousarray(a)
            if a.dtype == np.uint16:
                a = a.view(np.int16)
            return torch.from_numpy(a).to(dev)

        self.idx = torch.empty((m, k), dtype=torch.int32, device=dev)
        self.L.init_indices(self.idx, 1000 * cfg.index + wl.STREAM_IDX)
        self.W = up(wl.gen_W(cfg))
        self.m1 = torch.zeros((m, k), dtype=torch.float32, device=dev)
        self.m2 = torch.zeros((m, k), dtype=torch.float32, device=dev)
        self.gW = torch.empty((m, k), dtype=torch.float32, device=dev)
        self.xs = [up(wl.gen_x(cfg, i)) for i in range(cfg.n_x_batches)]
        self.tg = [tuple(up(a) for a in wl.gen_targets(cfg, i)) for i in range(cfg.n_x_batches)]
        self.out = torch.empty((b, m), dtype=torch.float32, device=dev)     # g is written in place
        self.gx = torch.empty((b, d), dtype=torch.float32, device=dev)
        self.loss = torch.empty((1,), dtype=torch.float32, device=dev)
        self.seed = wl.redistribution_seed(cfg)
        self.scale = float(np.float32(1.0 / b))
        self.t = 0
        self.epoch = 0

    def _redistribute(self):
        cfg = self.cfg
        if self.wl.is_redistribution_step(cfg, self.t):
            self.L.redistribute(self.idx, self.W, self.m1, self.m2, cfg.fraction, self.seed, self.epoch)
            self.epoch += 1
            return True
        return False

    def step(self, ev=None):
        """The step as four separate calls, with an event between the calls when ev is a list."""
        hp, b, L = self.wl.ADAM, self.cfg.b, self.L
        self.t += 1
        x = self.xs[self.t % len(self.xs)]
        off, lab = self.tg[self.t % len(self.tg)]
        marks = []

        def mark():
            if ev is not None:
                e = self.torch.cuda.Event(enable_timing=True)
                e.record(self.stream)
                marks.append(e)
        mark()
        L.forward(x, self.idx, self.W, self.out, b); mark()
        L.bce_loss_grad(self.out, off, lab, self.scale, self.out, self.loss, b); mark()
        L.backward(self.out, x, self.idx, self.W, self.gW, self.gx, b); mark()
        L.adam_step(self.W, self.gW, self.m1, self.m2, self.t, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"]); mark()
        if self._redistribute():
            mark()
        if ev is not None:
            ev.append(marks)

    def fused_step(self):
        hp, b = self.wl.ADAM, self.cfg.b
        self.t += 1
        x = self.xs[self.t % len(self.xs)]
        off, lab = self.tg[self.t % len(self.tg)]
        self.L.train_step(x, self.idx, self.W, self.m1, self.m2, off, lab, 0, self.scale, self.t, hp["lr"], hp["beta1"],
                          hp["beta2"], hp["eps"], self.out, self.gW, self.gx, self.loss, b)
        self._redistribute()

    def timed(self, fn, n):
        """HIP-event time of n calls of fn on the launch stream, in ms per call."""
        e0, e1 = self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True)
        e0.record(self.stream)
        for _ in range(n):
            fn()
        e1.record(self.stream)
        self.torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    def close(self):
        self.L.close()
        for name in list(vars(self)):
            if name not in ("cfg", "torch", "wl", "t", "epoch"):
                setattr(self, name, None)
        self.torch.cuda.empty_cache()


CALLS = ["forward", "bce", "backward", "adam", "redistribute"]        # the step as separate calls
STAGES = ["forward", "bce", "backward", "adam"]                       # ... those that every step has
ALONE = ["backward_weight", "backward_input"]                         # the two products of usl_backward, each by its own call


def per_call_breakdown(B, steps):
    """The same steps as separate calls with an event between the calls: ms per call and per step; then each of the two
    backward products by its own entry point, on the gradient the last step left."""
    events = []
    B.step()
    sep = B.timed(lambda: B.step(events), steps)
    per_call = {c: [] for c in CALLS}
    for marks in events:
        for i in range(len(marks) - 1):
            per_call[CALLS[i]].append(marks[i].elapsed_time(marks[i + 1]))
    res = {c: (float(np.mean(v)) if v else None) for c, v in per_call.items()}
    x, b, n = B.xs[0], B.cfg.b, max(2, min(steps, 10))
    for name, fn in (("backward_weight", lambda: B.L.backward_weight(B.out, x, B.idx, B.gW, b)),
                     ("backward_input", lambda: B.L.backward_input(B.out, B.idx, B.W, B.gx, b))):
        fn()
        res[name] = B.timed(fn, n)
    return res, sep


def workload_summary(name, steps, warmup, torch, usl, wl):
    """One of the other configurations, reported like the headline one (shorter)."""
    cfg = wl.CONFIGS[name]
    B = Bench(cfg, torch, usl, wl)
    for _ in range(warmup):
        B.fused_step()
    torch.cuda.synchronize()
    ms = B.timed(B.fused_step, steps)
    call_ms, sep = per_call_breakdown(B, max(2, steps // 2))
    ab = algorithmic_bytes(cfg)
    res = {"config": "m=%d d=%d k=%d b=%d %s, redistribution of %.0f%% every %d steps"
                     % (cfg.m, cfg.d, cfg.k, cfg.b, cfg.storage, 100 * cfg.fraction, cfg.period),
           "steps": steps, "ms_per_step": round(ms, 4), "steps_per_s": round(1e3 / ms, 2),
           "algorithmic_GB_per_step": round(ab["step"] / 1e9, 4),
           "achieved_hbm_GBps": round(ab["step"] / (ms * 1e-3) / 1e9, 1),
           "hbm_frac_of_peak": round(ab["step"] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
           "separate_calls_ms_per_step": round(sep, 4),
           "call_ms": {c: (round(v, 4) if v is not None else None) for c, v in call_ms.items()},
           "call_frac_of_peak": {c: round(ab[c] / (call_ms[c] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4) for c in STAGES + ALONE},
           "bad_rows": B.L.validate_indices(B.idx), "redistributions": B.epoch}
    dom = max(STAGES, key=lambda c: call_ms[c] or 0.0)
    res["roofline"] = {"bound": "hbm", "kernel": "usl_" + dom, "ms_per_launch": round(call_ms[dom], 4),
                       "launches_in_call": launches_in_call(cfg, dom), "algorithmic_bytes": ab[dom],
                       "achieved": round(ab[dom] / (call_ms[dom] * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                       "frac": round(ab[dom] / (call_ms[dom] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                       "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name, {}).get(dom)}
    B.close()
    return res


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
                    help="skip the legs a default run at N=1 appends: ceilings, the other workloads, the "
                         "squared-hinge sweep and the prediction timing")
    ap.add_argument("--sqh-sweep", action="store_true",
                    help="also time the squared-hinge loss and the two backward calls on gradients with "
                         "0 / 90 / 99 / 99.9 %% exact zeros (implicit negative mining, Section 3.3)")
    ap.add_argument("--separate-calls", action="store_true",
                    help="time the step as four separate calls instead of usl_train_step")
    ap.add_argument("--predict", action="store_true",
                    help="also time prediction (Section 2): top-5 labels of every score row and the P@k hit counts")
    ap.add_argument("--ceilings", action="store_true",
                    help="also run the library's measurement kernels (HBM streams, LDS gathers, L2 to LDS row "
                         "copies, L2 piece gathers) and relate the step to them")
    ap.add_argument("--other-workloads", action="store_true",
                    help="also report the configurations the headline is not quoted on (medium, large_wide, stress)")
    ap.add_argument("--traffic-kib", type=float, default=None,
                    help="HBM KiB per launch of the dominant kernel from rocprofv3 --pmc (FETCH+WRITE, scaled)")
    args = ap.parse_args()
    if not args.no_extras and not args.no_cpu_baseline and args.workload == "large":
        args.sqh_sweep = args.predict = args.ceilings = args.other_workloads = True
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
    B = Bench(cfg, torch, usl, wl)
    L, stream = B.L, B.stream
    idx, W, gW, gx, out, loss, xs, tg, scale = B.idx, B.W, B.gW, B.gx, B.out, B.loss, B.xs, B.tg, B.scale

    timed_step = B.step if args.separate_calls else B.fused_step
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
    t_wall0 = time.perf_counter()
    ms_per_step = B.timed(timed_step, args.steps)
    wall_ms = (time.perf_counter() - t_wall0) * 1e3
    loss_value = float(loss.item())
    call_ms, separate_ms = per_call_breakdown(B, args.steps)
    n_bad = L.validate_indices(idx)
    calls = CALLS
    ab = algorithmic_bytes(cfg)
    steps_per_s = 1e3 / ms_per_step
    # the dominant call and its roofline position (algorithmic bytes / measured time)
    dom = max(STAGES, key=lambda c: call_ms[c] or 0.0)
    dom_gbps = ab[dom] / (call_ms[dom] * 1e-3) / 1e9
    traffic = MEASURED_TRAFFIC_BYTES.get(cfg.name, {}).get(dom)
    if args.traffic_kib is not None:
        traffic = args.traffic_kib * 1024
    dom_kernels = KERNELS_OF_CALL["backward_one_pass" if dom == "backward" and one_pass_windows(cfg) else dom]
    roof = {"bound": "hbm", "kernel": "usl_%s: %s" % (dom, dom_kernels),
            "achieved": round(dom_gbps, 1), "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": round(dom_gbps / HBM_PEAK_GBPS, 4),
            "ms_per_launch": round(call_ms[dom], 4), "launches_in_call": launches_in_call(cfg, dom),
            "algorithmic_bytes": ab[dom],
            "traffic": traffic,
            "one_pass_lower_bound_bytes": ab["backward_one_pass_lower_bound"] if dom == "backward" else None,
            "note": "dominant call of the step (usl_train_step runs the same kernels, except that Adam takes the weight "
                    "gradient from where k_both_lds left it and k_unstage is not needed); achieved = algorithmic bytes "
                    "of the call (for usl_backward: of the two separate products it stands for) / HIP-event time of "
                    "the call on the launch stream, which covers launches_in_call "
                    "kernel launches (per-kernel durations: profiles/train_step_*_kernel_trace.txt); traffic = HBM "
                    "bytes per call from rocprofv3 counters (profiles/train_step_*_hbm_bytes.txt), measured offline"}
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
        "call_GBps": {c: round(ab[c] / (call_ms[c] * 1e-3) / 1e9, 1) for c in STAGES + ALONE},
        "wall_ms_per_step": round(wall_ms / args.steps, 4),
        "timed_path": ("separate calls: usl_forward, usl_bce_loss_grad, usl_backward, usl_adam_step"
                       if args.separate_calls else "usl_train_step (the same stages in one call)")
                      + ", usl_redistribute on its schedule",
        "separate_calls_ms_per_step": round(separate_ms, 4),
        "loss": loss_value, "bad_rows": n_bad, "redistributions": B.epoch,
        "roofline": roof,
    }
    if args.ceilings:
        try:
            from paper_2306_03725_amd import ceilings
            c = ceilings.run()
            cu, ghz = c["compute_units"], c["clock_GHz"]
            # one LDS gather per (instance, connection) and product; the two backward products share theirs where
            # usl_backward takes its one-pass form
            products = 2.0 if one_pass_windows(cfg) else 3.0
            gathers = products * b * m * k
            gather_rate = c["lds_gather_b32_conflict_free_lanes_per_clk_cu"] * cu * ghz * 1e9
            es = 2 if cfg.storage == "bf16" else 4
            # every product stages its rows into the LDS of every workgroup: per product, label (or feature)
            # blocks of 2048 x batch rows x row bytes
            copy_bytes = products * (-(-m // 2048)) * b * d * es
            t_gather = gathers / gather_rate * 1e3
            t_copy = copy_bytes / (c["l2_to_lds_row_copy_aggregate_GBps"] * 1e9) * 1e3
            t_hbm = ab["step"] / (c["hbm_copy_GBps_read_plus_write"] * 1e9) * 1e3
            res["ceilings"] = {k_: round(v, 3) for k_, v in c.items()}
            roof["gather_frac"] = round(t_gather / ms_per_step, 4)
            roof["gather_note"] = ("%d*b*m*k LDS gathers per step at the measured conflict-free ds_read_b32 rate "
                                   "would take %.3f ms; staging the rows those gathers read, at the measured L2 to "
                                   "LDS copy rate, %.3f ms; the step's algorithmic HBM bytes at the measured copy "
                                   "rate, %.3f ms; these three do not overlap inside a product kernel"
                                   % (int(products), t_gather, t_copy, t_hbm))
            roof["measured_ceilings_frac"] = round((t_gather + t_copy + t_hbm) / ms_per_step, 4)
        except Exception as exc:   # the headline line must survive a failure of an appended leg
            res["ceilings"] = {"error": repr(exc)}
    if args.sqh_sweep:
        try:
            # Synthetic stand-in for the gradient of a trained model under the squared hinge loss: the
            # scores' own gradient with a seeded share of entries forced to exactly zero.
            def timed(fn, reps=5):
                for _ in range(3):     # the library learns from finished calls whether to expect a sparse gradient
                    fn()
                    torch.cuda.synchronize()
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
            if cfg.storage == "f32":
                # The whole step under the squared hinge loss on a layer whose easy negatives are already separated
                # (stand-in for a trained model: all weights negative and large on non-negative activations, so
                # every score of a negative lies below -1 and only the positives keep a gradient).
                W_easy = -(W.abs() * 8.0 + 0.5)
                m1e, m2e = torch.zeros_like(W_easy), torch.zeros_like(W_easy)
                hp = wl.ADAM
                tt = [0]

                def easy_step():
                    tt[0] += 1
                    L.train_step(x0, idx, W_easy, m1e, m2e, off0, lab0, 1, scale, tt[0], hp["lr"], hp["beta1"],
                                 hp["beta2"], hp["eps"], gbuf, gW, gx, loss, b)
                sweep["train_step_easy_negatives"] = {
                    "ms_per_step": round(timed(easy_step, 10), 4),
                    "nonzero_share": round(float((gbuf != 0).float().mean().item()), 6),
                    "note": "usl_train_step with loss_kind = 1 (squared hinge), no redistribution; the step with "
                            "binary cross-entropy on the same shapes is ms_per_step above"}
                del W_easy, m1e, m2e
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
    B.close()
    del L, idx, W, gW, gx, out, loss, xs, tg
    torch.cuda.empty_cache()
    if args.other_workloads:
        res["workloads"] = {}
        for name, steps in (("medium", 50), ("large_wide", 10), ("stress", 4)):
            if name == cfg.name:
                continue
            try:
                res["workloads"][name] = workload_summary(name, steps, 2, torch, usl, wl)
            except Exception as exc:   # the headline line must survive a failure of an appended leg
                res["workloads"][name] = {"error": repr(exc)}
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
