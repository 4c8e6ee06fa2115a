#!/usr/bin/env python3
"""Benchmark of one GPU's share of a transformer layer's training step (forward + backward)
through libgx on MI355X.  Prints one JSON line.

A step is one pass of the whole hot path over one batch of seeded synthetic input already
resident in HBM: all blocks and micro-batches of the chosen workload, forward and backward.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0       # MI355X dense bf16 matrix peak (published)
PEAK_F32_TFLOPS = 157.3


def model_flops(sh, blocks, mbs):
    """Model FLOPs of forward + backward: the four projections plus causal attention counted on
    the unmasked pairs; backward is twice the forward; recomputation is not counted."""
    T, H, Hl, Fl = sh.tokens, sh.hidden, sh.hidden_local, sh.ffn_local
    fwd = 2.0 * T * H * 3 * Hl + 2.0 * T * Hl * H + 4.0 * T * H * Fl
    fwd += 4.0 * sh.micro_batch * sh.local_heads * sh.head_dim * sh.seq * (sh.seq + 1) / 2.0
    return 3.0 * fwd * blocks * mbs


def gemm_flops_by_class(sh, accumulate, wgrad_bf16=False):
    """Kernel class -> list of 2*M*N*K for the GEMM launches of one layer pass (fwd + bwd)."""
    T, H, Hl, Fl = sh.tokens, sh.hidden, sh.hidden_local, sh.ffn_local
    f = lambda m, n, k: 2.0 * m * n * k
    wg = (122 if accumulate else 120) if wgrad_bf16 else (126 if accumulate else 125)
    return {101: [f(T, 3 * Hl, H)], 102: [f(T, H, Hl), f(T, H, Fl)], 103: [f(T, Fl, H)],
            wg: [f(Fl, H, T), f(H, Fl, T), f(Hl, H, T), f(H, 3 * Hl, T)],
            114: [f(T, Fl, H)], 110: [f(T, H, Fl), f(T, Hl, H), f(T, H, 3 * Hl)]}


# HBM-side traffic of the dominant kernel class, measured with two rocprofv3 --pmc runs (FETCH_SIZE,
# then WRITE_SIZE; commands and per-kernel readings in profiles/), scaled by what the same counters
# read for --calibrate-copy's 256 MiB + 256 MiB elementwise copy.  The figure only holds for the
# kernel source it was measured on: `source_sha256` is the hash of csrc/gemm_bf16.hip at that time.
MEASURED_TRAFFIC = {
    # FETCH_SIZE x 1.9997 (copy calibration) + WRITE_SIZE x 1.0, averaged over the class's 4 launches per step:
    # dW2, dW1, dWqkv (256x256 tiles) 257.4 MB per launch on average, dWo (128x128 tiles) 117.5 MB
    ("C3", "gemm_tn_f32"): {"bytes_per_launch": 222.4e6, "algorithmic_bytes_per_launch": 109.1e6,
                            "source_sha256": "5ae1b3f5cd749b6cd072dc470d5479fc283f66a8369dd5040c428d379c02bfb6"},
}


def measured_traffic(workload, kernel):
    import hashlib
    m = MEASURED_TRAFFIC.get((workload, kernel))
    if not m:
        return None
    src = os.path.join(ROOT, "paper_2504_03662_amd", "csrc", "gemm_bf16.hip")
    if hashlib.sha256(open(src, "rb").read()).hexdigest() != m["source_sha256"]:
        return None
    return m["bytes_per_launch"]


class ClockPowerSampler:
    """Samples the shader clock (the starred line of amdgpu's pp_dpm_sclk) and the socket power (hwmon
    power1_average or power1_input, microwatts) from sysfs in a thread while a region runs.  Reads
    nothing but those files; reports null when the box does not expose them to this user."""

    def __init__(self, period_s=0.01):
        import glob
        self.period = period_s
        self.freq = self.power = None
        for dev in sorted(glob.glob("/sys/class/drm/card*/device")):
            f = os.path.join(dev, "pp_dpm_sclk")
            if self._sclk(f) is None:
                continue
            self.freq = f
            for q in sorted(glob.glob(os.path.join(dev, "hwmon/hwmon*/power1_average"))) + \
                    sorted(glob.glob(os.path.join(dev, "hwmon/hwmon*/power1_input"))):
                if self._number(q) is not None:
                    self.power = q
                    break
            break
        self.samples = []

    @staticmethod
    def _number(path):
        try:
            with open(path) as fh:
                return float(fh.read().strip())
        except (OSError, ValueError):
            return None

    @staticmethod
    def _sclk(path):
        """MHz of the current level: the line that ends in '*', e.g. '1: 1530Mhz *'."""
        try:
            with open(path) as fh:
                for line in fh:
                    if line.rstrip().endswith("*"):
                        return float(line.split(":")[1].lower().replace("mhz", "").replace("*", "").strip())
        except (OSError, ValueError, IndexError):
            pass
        return None

    def __enter__(self):
        import threading
        self._stop = threading.Event()

        def loop():
            while not self._stop.is_set():
                self.samples.append((self._sclk(self.freq), self._number(self.power) if self.power else None))
                self._stop.wait(self.period)
        self._t = threading.Thread(target=loop, daemon=True)
        if self.freq:
            self._t.start()
        return self

    def __exit__(self, *exc):
        self._stop.set()
        if self.freq:
            self._t.join()

    def summary(self):
        if not self.freq or not self.samples:
            return None
        f = [a for a, _ in self.samples if a]
        w = [b / 1e6 for _, b in self.samples if b]
        out = {"samples": len(self.samples), "source": [self.freq] + ([self.power] if self.power else [])}
        if f:
            out.update(sclk_mhz_min=min(f), sclk_mhz_mean=sum(f) / len(f), sclk_mhz_max=max(f))
        if w:
            out.update(power_w_min=min(w), power_w_mean=sum(w) / len(w), power_w_max=max(w))
        return out


def hbm_bound_figures(kernels, sh, both_phases=True):
    """Adds GB/s against the 8 TB/s HBM peak to the bandwidth-bound kernel classes of one block pass
    (algorithmic bytes: every operand read once, every result written once) and TFLOP/s against the
    matrix peak to the attention classes (causal attention counted on the unmasked pairs; the
    backward pass is 2.5 times the forward)."""
    T, H, Hl = sh.tokens, sh.hidden, sh.hidden_local
    e = 2 if sh.dtype == "bf16" else 4
    peak = PEAK_BF16_TFLOPS if sh.dtype == "bf16" else PEAK_F32_TFLOPS
    per_launch = {"ln_fwd": 2.0 * T * H * e,                 # x in, y out (statistics negligible)
                  "ln_bwd": 4.0 * T * H * e,                 # dy, x, residual gradient in, dx out
                  "colsum": None}
    for name, k in kernels.items():
        b = per_launch.get(name)
        if b:
            k["algorithmic_bytes_per_launch"] = b
            k["GB/s"] = b / (k["avg_ms"] * 1e-3) / 1e9
            k["frac_of_hbm_peak"] = k["GB/s"] / 8000.0
    attn = 4.0 * sh.micro_batch * sh.local_heads * sh.head_dim * sh.seq * (sh.seq + 1) / 2.0
    for name, mult in (("attn_fwd", 1.0), ("attn_bwd", 2.5)):
        if name in kernels:
            k = kernels[name]
            k["TFLOP/s"] = attn * mult / (k["avg_ms"] * 1e-3) / 1e12
            k["frac_of_mfma_peak"] = k["TFLOP/s"] / peak


def run_peaks():
    """Measured ceilings of this machine, as one JSON line: the register-only MFMA loop and the plain copy
    of the library's measurement hooks, and, as context, the vendor library's GEMM (through
    torch.matmul) on the C3 layer's product shapes with the same kind of operands (N(0,1) activations,
    N(0, 0.02^2) weights) and with constant operands."""
    import torch
    from paper_2504_03662_amd import binding as gx
    st = torch.cuda.current_stream().cuda_stream
    scratch = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    out = {"mfma_loop_tflops": gx.peak_mfma(scratch, 20, st)}
    n = 1 << 29
    src = torch.ones(n // 4, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    out["copy_gbps_read_plus_write"] = gx.peak_copy(src, dst, n, 20, st)
    del src, dst

    def timed(fn, reps=30):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    table = []
    torch.manual_seed(0)
    for (M, N, K) in [(4096, 4096, 4096), (4096, 3072, 4096), (4096, 4096, 1024), (4096, 1024, 4096)]:
        for kind in ("normal", "ones"):
            mk = (lambda *d: torch.randn(*d, device="cuda:0", dtype=torch.bfloat16)) if kind == "normal" else \
                 (lambda *d: torch.ones(*d, device="cuda:0", dtype=torch.bfloat16))
            a, at = mk(M, K), mk(K, M)
            b, bt = mk(K, N) * (0.02 if kind == "normal" else 1.0), mk(N, K) * (0.02 if kind == "normal" else 1.0)
            fl = 2.0 * M * N * K
            table.append({"M": M, "N": N, "K": K, "operands": kind,
                          "NN": fl / timed(lambda: torch.matmul(a, b)) / 1e9,
                          "NT": fl / timed(lambda: torch.matmul(a, bt.t())) / 1e9,
                          "TN": fl / timed(lambda: torch.matmul(at.t(), b)) / 1e9})
    out["vendor_gemm_tflops"] = table
    print(json.dumps(out))


CLASS_NAMES = {1: "ln_fwd", 2: "ln_bwd", 3: "attn_fwd", 4: "attn_bwd", 5: "colsum", 6: "dropout",
               101: "gemm_nn_bias", 102: "gemm_nn_resid", 103: "gemm_nn_gelu", 110: "gemm_nt_store",
               114: "gemm_nt_dgelu", 125: "gemm_tn_f32", 126: "gemm_tn_f32_acc",
               120: "gemm_tn_bf16", 122: "gemm_tn_bf16_acc"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps (default: about 0.27 s of them, at least 20 and at most 200; a region of "
                         "20 steps of 1.3 ms reads 0.7 %% low, the two ends of the region being what they are)")
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C3", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--serial", action="store_true",
                    help="queue the backward pass on one stream (no side-stream overlap) in the timed region "
                         "too; the per-kernel timing pass always runs that way")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain elementwise copy of 256 MiB (read) + 256 MiB (write), as the "
                         "known-size reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--wgrad-bf16", action="store_true",
                    help="variant: weight-matrix gradients written as bf16 (GX_WGRAD_BF16) instead of fp32; "
                         "recorded in config.weight_grad")
    ap.add_argument("--dropout", type=int, default=0, metavar="P256",
                    help="variant: dropout of the attention probabilities and of each half's output with "
                         "probability P256/256 (GX_DROPOUT); recorded in config.dropout_256ths")
    ap.add_argument("--zero-operands", action="store_true",
                    help="diagnostic, not a benchmark: run the same step on all-zero activations, upstream "
                         "gradients and parameters (every product multiplies zeros), which shows how fast the same kernels "
                         "and launch sequence run when operand switching activity does not hold the clock down; "
                         "recorded in \"data\"")
    ap.add_argument("--peaks", action="store_true",
                    help="instead of the benchmark: measure this box's ceilings (register-only MFMA loop, plain "
                         "copy, the vendor library's GEMM on the layer's product shapes) and print them as JSON")
    ap.add_argument("--sustain-seconds", type=float, default=2.0,
                    help="before the per-kernel pass and the timed region, run steps back to back for this long while "
                         "sampling shader clock and socket power (reported under \"sustained\"; 0 to skip)")
    ap.add_argument("--neighbours", action="store_true",
                    help="also time the layer step's memory-bound neighbours at this workload's shapes (AdamW "
                         "update of the rank's parameters, slicing the rank's shard out of the whole block and "
                         "merging it back) and report them under \"neighbours\"")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU's share on one GPU: run it with --gpus 1 "
                 "(the library runs no collective; there is no multi-GPU path to time)")

    import torch
    from paper_2504_03662_amd import binding as gx
    from paper_2504_03662_amd import inputs as I
    from paper_2504_03662_amd.runtime import DeviceStack, StageSchedule, one_f_one_b, to_device

    gx.lib()                                         # fails loudly when the HIP library is missing
    gx.set_overlap(not args.serial)
    if not torch.cuda.is_available():
        sys.exit("bench.py needs an MI355X: no GPU is visible")
    if args.peaks:
        run_peaks()
        return
    shape, blocks, mbs = I.WORKLOADS[args.workload]
    if args.dropout:
        shape = shape.with_(drop_attn=args.dropout, drop_hidden=args.dropout, drop_seed=20250403)
    case = {"C1": 1, "C2": 2, "C3": 3, "C4": 4, "C5": 5}[args.workload]
    plist = [I.rank_params(shape, case=case, block=k) for k in range(blocks)]
    stack = DeviceStack(shape, plist, wgrad_bf16=args.wgrad_bf16)
    del plist
    acts = [I.activations(shape, case=case, micro_batch_index=m) for m in range(mbs)]
    xs = [to_device(a[0], shape.dtype) for a in acts]
    dys = [to_device(a[1], shape.dtype) for a in acts]
    if args.zero_operands:
        for t in xs + dys + [w for layer in stack.layers for w in layer.params.values()]:
            t.zero_()
    pipelined = mbs > 1
    schedule = one_f_one_b(mbs, 3) if pipelined else [("F", 0), ("B", 0)]

    # pipelined stage: full activation recomputation, gradients summed over micro-batches; forward
    # and backward passes of different micro-batches are issued on two streams (unless --serial)
    runner = StageSchedule(stack, mbs, overlap=pipelined and not args.serial)

    def step():
        runner.run(schedule, xs, dys, recompute=pipelined)

    if args.calibrate_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 1.0, out=dst)              # one vectorized elementwise kernel: 256 MiB in, 256 MiB out
        torch.cuda.synchronize()
        del src, dst
    # Order of the measurements: (1) back-to-back steps for a couple of seconds, (2) the per-kernel
    # pass, (3) the warm-up steps and the timed region.  From idle the chip needs some 50 to 100
    # steps (about 0.1 s) before step times settle (measured: 1.53 ms for the first steps, 1.40 after
    # ten, 1.35 from about step 80 on, while the shader clock drifts DOWN from 2.3 to 2.04 GHz as the
    # power limit takes hold), so a timed region that follows five warm-up steps would report the
    # transient and not what a training job sees; (1) is that steady state measured directly and
    # reported under "sustained", and it leaves the chip in it for (2) and (3).
    sustained = None
    if args.sustain_seconds > 0:
        step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(8):
            step()
        torch.cuda.synchronize()
        est_ms = (time.perf_counter() - t1) * 1e3 / 8
        if args.steps is None:
            args.steps = max(20, min(200, int(round(270.0 / est_ms))))
        n_sus = max(args.steps, int(args.sustain_seconds * 1e3 / est_ms))
        with ClockPowerSampler(0.01) as sus_sampler:
            t1 = time.perf_counter()
            for i in range(n_sus):
                step()
                if i % 64 == 63:
                    torch.cuda.synchronize()        # bound the launch queue
            torch.cuda.synchronize()
            sus_ms = (time.perf_counter() - t1) * 1e3 / n_sus
        sustained = {"steps": n_sus, "ms_per_step": sus_ms, "clock_power": sus_sampler.summary()}
    if args.steps is None:
        args.steps = 20
    # per-kernel-class durations from HIP events on the launch stream: the same work with the
    # backward pass queued serially (kernels that overlap share the chip, so only a kernel that has
    # it alone can be held against the roofline).
    torch.cuda.synchronize()
    gx.set_overlap(False)
    serial = StageSchedule(stack, mbs, overlap=False)

    def step_serial():
        serial.run(schedule, xs, dys, recompute=pipelined)

    step_serial()
    gx.prof_enable(True)
    launches_per_step = None
    rec = []
    for _ in range(max(1, min(args.steps, 8))):
        step_serial()
        got = gx.prof_collect()
        launches_per_step = len(got)
        rec += got
    gx.prof_enable(False)
    gx.set_overlap(not args.serial)
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    with ClockPowerSampler(0.002) as timed_sampler:
        t0 = time.perf_counter()
        for i in range(args.steps):
            step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
    # median and minimum per step come from a second pass of as many steps with an event after each
    # (an event between steps costs the step about half a percent, so the timed region has none)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    marks[0].record()
    for i in range(args.steps):
        step()
        marks[i + 1].record()                       # on the stream every step starts from and joins back to
    torch.cuda.synchronize()
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    flops = model_flops(shape, blocks, mbs)
    tflops = flops / (ms * 1e-3) / 1e12
    peak = PEAK_BF16_TFLOPS if shape.dtype == "bf16" else PEAK_F32_TFLOPS

    by = {}
    for c, t in rec:
        by.setdefault(c, []).append(t)
    total_ms = sum(sum(v) for v in by.values())
    kernels = {CLASS_NAMES.get(c, str(c)): {"launches_per_step": len(v) * launches_per_step // len(rec),
                                            "avg_ms": sum(v) / len(v), "share": sum(v) / total_ms}
               for c, v in sorted(by.items(), key=lambda kv: -sum(kv[1]))}
    gemm_fl = gemm_flops_by_class(shape, pipelined, args.wgrad_bf16)
    dom = max((c for c in by if c >= 100), key=lambda c: sum(by[c]))
    pair = {125: 126, 126: 125, 120: 122, 122: 120}                      # store / accumulate forms of one product
    fl = gemm_fl.get(dom) or gemm_fl.get(pair.get(dom))                  # first micro-batch overwrites
    avg_ms = sum(by[dom]) / len(by[dom])
    if dom in pair and pipelined:
        both = by.get(dom, []) + by.get(pair[dom], [])
        avg_ms = sum(both) / len(both)
    flops_per_launch = sum(fl) / len(fl)
    achieved = flops_per_launch / (avg_ms * 1e-3) / 1e12
    gemm_ms = sum(sum(v) for c, v in by.items() if c >= 100)
    gemm_tflops = sum(sum(v) for v in gemm_fl.values()) * blocks * mbs * (len(rec) / launches_per_step) \
        / (gemm_ms * 1e-3) / 1e12 if not pipelined else None
    roofline = {"bound": "mfma", "kernel": CLASS_NAMES.get(dom, str(dom)), "achieved": achieved, "peak": peak,
                "unit": "TFLOP/s", "frac": achieved / peak,
                "traffic": measured_traffic(args.workload, CLASS_NAMES.get(dom, str(dom))),
                "traffic_source": "stored from profiles/ (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE); null when the "
                                  "kernel source has changed since the counters were taken",
                "avg_launch_ms": avg_ms,
                "flops_per_launch": flops_per_launch, "all_gemms_tflops": gemm_tflops}

    hbm_bound_figures(kernels, shape)
    if sustained:
        sustained["value"] = flops / (sustained["ms_per_step"] * 1e-3) / 1e12
    out = {"metric": "layer fwd+bwd TFLOP/s per GPU", "value": tflops, "unit": "TFLOP/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
           "ms_per_step_median": per_step[len(per_step) // 2], "ms_per_step_min": per_step[0],
           "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": shape.dtype,
           "data": "zeros (clock diagnostic, not a benchmark)" if args.zero_operands else "synthetic",
           "config": {"workload": args.workload, "hidden": shape.hidden, "heads": shape.heads, "ffn": shape.ffn,
                      "tp_attn": shape.tp_attn, "tp_ffn": shape.tp_ffn, "tp_rank": shape.tp_rank, "seq": shape.seq,
                      "micro_batch": shape.micro_batch, "blocks": blocks, "micro_batches": mbs,
                      "schedule": ("1F1B, full recompute, forward and backward passes on two streams"
                                   if runner.overlap else "1F1B, full recompute") if pipelined else "fwd then bwd",
                      "backward_overlap": not args.serial, "weight_grad": "bf16" if args.wgrad_bf16 else "f32",
                      "dropout_256ths": args.dropout},
           "frac_of_mfma_peak": tflops / peak,
           "tokens_per_s_per_layer": shape.tokens * blocks * mbs / (ms * 1e-3),
           "model_tflop_per_step": flops / 1e12,
           "roofline": roofline, "kernels": kernels,
           "clock_power_timed_region": timed_sampler.summary(), "sustained": sustained,
           "order": "sustained run, per-kernel pass, warm-up steps, timed region, per-step pass" if sustained else
                    "per-kernel pass, warm-up steps, timed region, per-step pass"}

    if args.neighbours:
        out["neighbours"] = neighbours(shape, stack, max(3, min(args.steps, 20)))
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, case)
    print(json.dumps(out))


def neighbours(shape, stack, reps):
    """HBM-bound passes next to the layer step, timed with HIP events on the current stream and held
    against the 8 TB/s HBM peak by their algorithmic bytes: AdamW reads w, m, v, g and writes w, m, v
    (fp32) plus the bf16 copy = 30 B per element; a shard transition reads and writes each element of
    the rank's shard once."""
    import torch
    from paper_2504_03662_amd import binding as gx
    from paper_2504_03662_amd import inputs as I
    dev = "cuda:0"
    st = torch.cuda.current_stream().cuda_stream
    n = sum(int(t.numel()) for t in stack.layers[0].params.values())
    w, m, v, g = (torch.randn(n, device=dev) * s for s in (0.02, 1e-3, 1e-3, 1e-2))
    v = v * v + 1e-8
    out = torch.empty(n, dtype=torch.bfloat16, device=dev)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    step = [0]

    def adam():
        step[0] += 1
        gx.adamw_step(n, w, m, v, g, out, gx.GX_BF16, step=step[0], lr=1e-4, weight_decay=0.01, stream=st)

    t_adam = timed(adam)
    res = {"adamw": {"elements": n, "ms": t_adam, "GB/s": 30.0 * n / t_adam / 1e6, "frac_of_hbm_peak": 30.0 * n / t_adam / 1e6 / 8000.0}}
    del w, m, v, g, out
    H, F = shape.hidden, shape.ffn
    e = 2 if shape.dtype == "bf16" else 4
    tdt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
    dims = dict(ln1_g=(H,), ln1_b=(H,), w_qkv=(H, 3 * H), b_qkv=(3 * H,), w_o=(H, H), b_o=(H,),
                ln2_g=(H,), ln2_b=(H,), w_fc1=(H, F), b_fc1=(F,), w_fc2=(F, H), b_fc2=(H,))
    whole_bytes = sum(e * int(torch.Size(d).numel()) for d in dims.values())
    if whole_bytes <= 8 << 30:
        whole = {k: torch.zeros(d, dtype=tdt, device=dev) for k, d in dims.items()}
        shard = stack.layers[0].params
        cfg = gx.make_cfg(H, shape.heads, F, shape.tp_attn, shape.tp_ffn, shape.tp_rank, 1, 1,
                          gx.GX_BF16 if shape.dtype == "bf16" else gx.GX_F32, 3)
        sbytes = sum(int(t.numel()) * e for t in shard.values())
        t_merge = timed(lambda: gx.params_merge(cfg, shard, whole, stream=st))
        tmp = {k: torch.empty_like(t) for k, t in shard.items()}
        t_slice = timed(lambda: gx.params_slice(cfg, whole, tmp, stream=st))
        for name, t in (("params_merge", t_merge), ("params_slice", t_slice)):
            res[name] = {"shard_bytes": sbytes, "ms": t, "GB/s": 2.0 * sbytes / t / 1e6,
                         "frac_of_hbm_peak": 2.0 * sbytes / t / 1e6 / 8000.0}
    return res


def cpu_baseline(shape, case):
    """The fp64 NumPy oracle, as it stands, timed on the host on a bounded sample of the same
    workload: one block at the workload's own shard shape and micro-batch, forward + backward,
    repeated until about 10 s of CPU time have been spent (at most 4 times)."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import layer as O
    from paper_2504_03662_amd import inputs as I

    params = I.rank_params(shape, case=case, block=0)
    x, dy = I.activations(shape, case=case)
    fl = O.model_flops(shape)
    reps, spent = 0, 0.0
    while reps < 4 and spent < 10.0:
        t0 = time.perf_counter()
        fwd = O.layer_fwd(shape, params, x)
        O.layer_bwd(shape, params, dy, fwd["cache"])
        spent += time.perf_counter() - t0
        reps += 1
        del fwd
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    return {"value": fl * reps / spent / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": f"one block of the workload's shard shape (seq {shape.seq}, micro-batch {shape.micro_batch}), "
                      f"fwd+bwd x{reps}, fp64 NumPy ({fl * reps / 1e9:.0f} GFLOP in {spent:.1f} s)",
            "seconds": spent, "host_cpus": os.cpu_count()}


if __name__ == "__main__":
    main()
