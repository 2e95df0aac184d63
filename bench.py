#!/usr/bin/env python3
"""Benchmark of the per-example clipping hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch of the chosen
configuration: squared norms of every layer (accumulated over layers), clip
factors, the clipped gradient sum of every layer, and Gaussian noise where the
configuration asks for it.  Inputs are resident in HBM before timing starts.

Prints ONE JSON line (see README/DESIGN for the fields).  Only one GPU is
supported: --gpus above 1 exits with a message.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

# HBM bytes per launch of the dominant kernel, from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) of
# `bench.py --calib-copy`, scaled by what the same counters read for the 1 GiB copy (see profiles/).
# None until measured for the current kernels.
MEASURED_TRAFFIC = {
    # the clipped-sum phase of one step: the launch that takes all four layers (995.3 MB read, 198.2 MB written) and
    # the launch that folds their K slices (198.2 MB read, 28.3 MB written) (profiles/transformer_hbm_traffic.md)
    "transformer": 1420.0e6,
}

PEAK_HBM_GBS = 8000.0
PEAK_MFMA_TFLOPS = {"bf16": 2500.0, "f16": 2500.0, "f32": 157.3, "f8": 5000.0, "f8e4m3": 5000.0, "f8e5m2": 5000.0}
SPINUP_S = 0.04          # untimed busy time in front of every timed loop (see time_steps)


def to_dev(x, torch, f8=None):
    """f8: torch dtype of uint8 bit patterns (the two 8-bit formats are told apart by the workload's dtype name)."""
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
    if x.dtype == np.uint8:
        return torch.from_numpy(x).cuda().view(f8)
    return torch.from_numpy(x).cuda()


def f8_torch_types(dtype, torch):
    from paper_2009_03106_amd import workloads as wl
    t = {"f8e4m3": torch.float8_e4m3fn, "f8e5m2": torch.float8_e5m2}
    sa, sg = wl.f8_formats(dtype)
    return t[sa], t[sg]


class Pipeline:
    """Device buffers and the call sequence for one configuration; nothing is allocated inside step()."""

    def __init__(self, w, layers_np, torch, dp, path="auto"):
        self.w, self.torch, self.dp, self.path = w, torch, dp, path
        ta, tg = f8_torch_types(w.dtype, torch) if w.dtype.startswith("f8") else (None, None)
        self.dev = [(to_dev(A, torch, ta), to_dev(G, torch, tg)) for A, G in layers_np]
        self.B = self.dev[0][0].shape[0]
        dt = {"f32": dp.DP_F32, "bf16": dp.DP_BF16, "f16": dp.DP_F16, "f8e4m3": dp.DP_F8_E4M3, "f8e5m2": dp.DP_F8_E5M2,
              "f8": dp.DP_F8_E4M3_E5M2}[w.dtype]
        self.s = torch.zeros(self.B, dtype=torch.float32, device="cuda")
        self.c = torch.zeros(self.B, dtype=torch.float32, device="cuda")
        self.grads = []
        # the layers' gradients lie one after the other in one flat buffer (the model's flat parameter gradient):
        # the noise is then one call over the whole buffer, whose offsets are the per-layer calls' running offsets
        sizes = [spec.d_in * spec.d_out for spec in w.layers]
        self.flat_grad = torch.zeros(sum(sizes), dtype=torch.float32, device="cuda")
        starts = np.concatenate([[0], np.cumsum(sizes)]).tolist()
        for li, spec in enumerate(w.layers):
            self.grads.append(self.flat_grad[starts[li]:starts[li + 1]].view(spec.d_in, spec.d_out))
        self.descs = dp.layer_descs(self.dev)
        order = sorted(range(len(self.dev)), key=lambda li: self.dev[li][0].shape[2] + self.dev[li][1].shape[2])
        self.dev_cg = [self.dev[li] for li in order]
        self.descs_cg = dp.layer_descs(self.dev_cg, [self.grads[li] for li in order], [starts[li] for li in order])
        self.ws_cg_all = torch.empty(max(16, dp.layers_clipped_workspace_bytes(self.descs_cg[0], self.B, dt)), dtype=torch.uint8, device="cuda")
        self.ws_layers = torch.empty(max(16, dp.layers_workspace_bytes(self.descs[0], self.B, dt, path)), dtype=torch.uint8, device="cuda")
        need = max(16, dp.layers_workspace_bytes(self.descs_cg[0], self.B, dt, path), self.ws_cg_all.numel())
        self.ws_step = self.ws_cg_all if need <= self.ws_cg_all.numel() else torch.empty(need, dtype=torch.uint8, device="cuda")

    def phase_sqnorm(self):
        # all layers in one call: the copy-pipeline Gram layers share a launch, dense layers share one, and the
        # launch that completes the norms writes the clip factors (a kernel of its own where no Gram launch does)
        self.dp.layers_sqnorm(self.dev, self.s, path=self.path, workspace=self.ws_layers, descs=self.descs,
                              C=self.w.C, clip=self.c)

    def phase_clip(self):
        pass                                                   # done by phase_sqnorm

    def phase_grad(self):
        # the layers that the norm phase read last first: their inputs are the likeliest to be still in the
        # Infinity Cache (the several-layers call runs the widest layers first); the noise of the flat gradient
        # buffer is added by the kernels that fold the K slices (by the noise kernel where there is one slice)
        self.dp.layers_clipped_grad(self.dev_cg, self.c, workspace=self.ws_cg_all, descs=self.descs_cg,
                                    noise_std=self.w.noise_std, seed=self.w.noise_seed)

    def phase_noise(self):
        pass                                                   # added in phase_grad

    def step(self, events=None):
        if events is None:
            # the whole step in one library call (dp_layers_step): the same launches as the two calls below
            self.dp.layers_step(self.descs_cg, self.w.C, self.s, self.c, self.ws_step, path=self.path,
                                noise_std=self.w.noise_std, seed=self.w.noise_seed)
            return
        if events is not None:
            events[0].record()
        self.phase_sqnorm()
        if events is not None:
            events[1].record()
        self.phase_clip()
        if events is not None:
            events[2].record()
        self.phase_grad()
        if events is not None:
            events[3].record()
        self.phase_noise()
        if events is not None:
            events[4].record()


def algorithmic_work(w, B):
    """Flops and HBM bytes per step that the method itself needs (no re-reads, no scratch)."""
    es = 2 if w.dtype in ("bf16", "f16") else (1 if w.dtype.startswith("f8") else 4)
    out = {"norm_flops": 0, "gemm_flops": 0, "norm_bytes": 0, "gemm_bytes": 0, "noise_bytes": 0}
    for spec in w.layers:
        T, di, do = spec.T, spec.d_in, spec.d_out
        if T == 1:
            out["norm_flops"] += 2 * B * (di + do)
        else:
            gram = T * (T + 1) * (di + do)
            direct = 2 * T * di * do
            out["norm_flops"] += B * min(gram, direct)
        out["gemm_flops"] += 2 * B * T * di * do
        out["norm_bytes"] += B * T * (di + do) * es + 4 * B
        out["gemm_bytes"] += B * T * (di + do) * es + 4 * di * do
        if w.noise_std > 0:
            out["noise_bytes"] += 8 * di * do
    return out


def time_steps(pipe, torch, steps, warmup):
    """(ms per step, ms per phase).  The step time is the wall clock around `steps` back-to-back steps between two
    device synchronisations, with nothing else in the stream; the phase times come from a second pass of the same
    number of steps with HIP events between the phases (the event records cost a few microseconds each, which is
    why they stay out of the pass that is timed as a whole)."""
    # After an idle period the chip's power management overshoots: from a cold start the second step of the
    # transformer configuration takes 0.79 ms, steps 4-6 about 1.05 ms, and the rate settles (0.80 ms) only after
    # some 25 steps = 20 ms.  A training run lives in the settled state, so the device is kept busy with untimed
    # steps for SPINUP_S seconds before the warm-up steps; the K timed steps then follow without a pause.
    t_spin = time.perf_counter()
    while time.perf_counter() - t_spin < SPINUP_S:
        for _ in range(4):
            pipe.step()
        torch.cuda.synchronize()
    for _ in range(warmup):
        pipe.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        pipe.step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(steps)]
    for k in range(steps):
        pipe.step(evs[k])
    torch.cuda.synchronize()
    phases = np.zeros(4)
    for k in range(steps):
        for p in range(4):
            phases[p] += evs[k][p].elapsed_time(evs[k][p + 1])
    return (t1 - t0) * 1e3 / steps, phases / steps      # ms per step, ms per phase


def time_steps_cold(pipe, torch, steps, flush):
    """Phase times with the caches emptied before every step: a 512 MB buffer (twice the 256 MB of Infinity
    Cache) is read between steps, so each step's first pass over A and G comes from HBM.  The flush only reads:
    a flush that writes leaves dirty lines whose write-back would be charged to the step that follows."""
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(steps)]
    for k in range(steps):
        flush.max()
        pipe.step(evs[k])
    torch.cuda.synchronize()
    phases = np.zeros(4)
    for k in range(steps):
        for p in range(4):
            phases[p] += evs[k][p].elapsed_time(evs[k][p + 1])
    return phases / steps


def measured_peaks(torch, dp):
    """What this part sustains, from the library's own probe kernels (include/dpclip_probes.h), each timed with HIP
    events over a launch of about 10 ms after the same spin-up as the steps: the matrix units with operands in
    registers (constant operands reach the published peak; pseudo-random ones, which is what streaming data looks
    like to the multipliers, make the part lower its clock), a plain read of 1 GiB (four times the last-level
    cache, so every pass comes from HBM), and the LDS reads of the Gram kernel (ds_read_b128) and of the
    clipped-sum kernels (ds_read_b64_tr_b16) with 8 waves per compute unit."""
    sink = torch.zeros(dp.PROBE_SINK_FLOATS, dtype=torch.float32, device="cuda")
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]

    def timed(launch, reps=3):
        t_spin = time.perf_counter()
        while time.perf_counter() - t_spin < SPINUP_S:
            launch()
            torch.cuda.synchronize()
        best, work = None, 0.0
        for _ in range(reps):
            ev[0].record()
            work = launch()
            ev[1].record()
            torch.cuda.synchronize()
            ms = ev[0].elapsed_time(ev[1])
            best = ms if best is None else min(best, ms)
        return work / (best * 1e-3), best

    out = {}
    for name, code, iters in (("bf16", dp.DP_BF16, 12000), ("f16", dp.DP_F16, 12000), ("f8_e4m3_e5m2", dp.DP_F8_E4M3_E5M2, 6000)):
        for rnd in (0, 1):
            rate, ms = timed(lambda: dp.probe_mfma(code, rnd, iters, sink))
            out[f"mfma_{name}_{'random' if rnd else 'constant'}_operands_tflops"] = rate / 1e12
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    rate, ms = timed(lambda: dp.probe_read(src, sink), reps=5)
    out["hbm_read_gbs"] = rate / 1e9
    small = src[: (96 << 20) // 4]
    rate, ms = timed(lambda: dp.probe_read(small, sink), reps=5)
    out["last_level_cache_read_gbs"] = rate / 1e9
    del src, small
    for name, kind in (("lds_read_b128", 0), ("lds_read_b64_tr_b16", 1)):
        rate, ms = timed(lambda: dp.probe_lds_read(kind, 20000, sink))
        out[f"{name}_gb_per_s_per_cu"] = rate / 1e9 / 256
    out["note"] = "probe kernels of libdpclip.so (dp_probe_*), best of 3-5 launches of about 10 ms each, HIP events"
    return out


def power_trace(pipe, torch, dp, seconds=2.0):
    """Socket power and shader clock (amdsmi, sampled every 100 ms by a thread) while each phase of the step, and
    each of the probe kernels, loops for `seconds`: tells whether a kernel runs at the part's clock limit or at its
    power limit.  The first half second of every loop (the transient) is left out of the means."""
    import threading
    import amdsmi
    amdsmi.amdsmi_init()
    h = amdsmi.amdsmi_get_processor_handles()[0]
    out = {"power_limit_w": amdsmi.amdsmi_get_power_info(h)["power_limit"] / 1e6}

    def during(work):
        rows, stop = [], threading.Event()

        def sample():
            while not stop.is_set():
                rows.append((time.perf_counter(), amdsmi.amdsmi_get_power_info(h)["current_socket_power"],
                             amdsmi.amdsmi_get_clock_info(h, amdsmi.AmdSmiClkType.GFX)["clk"]))
                time.sleep(0.1)
        th = threading.Thread(target=sample)
        t0 = time.perf_counter()
        th.start()
        n = 0
        while time.perf_counter() - t0 < seconds:
            work()
            n += 1
            torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        stop.set()
        th.join()
        kept = [r for r in rows if r[0] - t0 > 0.5] or rows
        return {"socket_power_w": float(np.mean([r[1] for r in kept])), "gfx_clock_mhz": float(np.mean([r[2] for r in kept])),
                "samples": len(kept), "rounds_per_s": n / dt}

    sink = torch.zeros(dp.PROBE_SINK_FLOATS, dtype=torch.float32, device="cuda")
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    out["idle"] = during(lambda: time.sleep(0.05))
    out["steps"] = during(lambda: [pipe.step() for _ in range(20)])
    out["steps"]["ms_per_step"] = 1e3 / (20 * out["steps"].pop("rounds_per_s"))
    out["sqnorm_phase"] = during(lambda: [pipe.phase_sqnorm() for _ in range(40)])
    out["sqnorm_phase"]["ms"] = 1e3 / (40 * out["sqnorm_phase"].pop("rounds_per_s"))
    out["clipped_grad_phase"] = during(lambda: [pipe.phase_grad() for _ in range(20)])
    out["clipped_grad_phase"]["ms"] = 1e3 / (20 * out["clipped_grad_phase"].pop("rounds_per_s"))
    for name, rnd in (("mfma_probe_random_operands", 1), ("mfma_probe_constant_operands", 0)):
        flops = dp.probe_mfma(dp.DP_BF16, rnd, 12000, sink)
        out[name] = during(lambda: dp.probe_mfma(dp.DP_BF16, rnd, 12000, sink))
        out[name]["tflops"] = flops * out[name].pop("rounds_per_s") / 1e12
    nbytes = dp.probe_read(src, sink)
    out["hbm_read_probe"] = during(lambda: [dp.probe_read(src, sink) for _ in range(10)])
    out["hbm_read_probe"]["gbs"] = 10 * nbytes * out["hbm_read_probe"].pop("rounds_per_s") / 1e9
    out["idle"].pop("rounds_per_s")
    return out


def cpu_baseline(name, sample_B, threads=None):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same workload."""
    from oracle import dp_oracle as orc
    from paper_2009_03106_amd import workloads as wl
    import contextlib
    limit = contextlib.nullcontext()
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        if threads is not None:
            limit = threadpool_limits(limits=int(threads))
        else:
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = 1 if threads is None else threads
    w, layers = wl.generate(name, B=sample_B)
    reps = 0
    with limit:
        t0 = time.perf_counter()
        while True:                                   # tiny configurations: repeat until the clock can see them
            orc.run_pipeline(layers, w.C, w.noise_std, w.noise_seed)
            reps += 1
            dt = time.perf_counter() - t0
            if dt > 0.2 or reps >= 200:
                break
    return {"value": sample_B * reps / dt, "unit": "examples/s", "cores": int(threads), "host_cpus": os.cpu_count(),
            "kind": "oracle",
            "sample": f"{name} configuration with B={sample_B} of {w.B} examples, all layers, float64, "
                      f"{reps} pass(es) in {dt:.2f} s wall, {int(threads)} BLAS thread(s)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="transformer")
    ap.add_argument("--path", default="auto", choices=["auto", "gram", "direct"])
    ap.add_argument("--dtype", default=None, choices=["f16", "f8", "f8e4m3", "f8e5m2"],
                    help="store the configuration's inputs in another type (not the headline run: profiles of the variants)")
    ap.add_argument("--batch", type=int, default=None, help="override the configuration's batch size (sweeps)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the short runs of the other configurations")
    ap.add_argument("--no-peaks", action="store_true", help="skip the probe kernels that measure what the part sustains")
    ap.add_argument("--peaks", action="store_true", help="only measure the peaks (probe kernels) and print them")
    ap.add_argument("--power", action="store_true",
                    help="only sample socket power and shader clock (amdsmi) while the phases and the probe kernels loop")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy (a kernel of known traffic) so that a rocprofv3 "
                         "--pmc run of this command can scale FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2009_03106_amd import dpclip as dp, workloads as wl
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    dp.load_library()

    if args.peaks:
        print(json.dumps({"measured_peaks": measured_peaks(torch, dp)}))
        return

    if args.calib_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    w, layers = wl.generate(args.workload, B=args.batch, dtype=args.dtype)
    if args.dtype is not None:
        w = dataclasses.replace(w, dtype=args.dtype)
    pipe = Pipeline(w, layers, torch, dp, args.path)
    del layers
    B = pipe.B
    if args.power:
        print(json.dumps({"workload": w.name, "dtype": w.dtype, "power": power_trace(pipe, torch, dp)}))
        return
    # the same K steps after W warm-up steps straight from an idle device, without the spin-up that time_steps puts
    # in front (the power management's start-up transient is inside this figure; it is reported, not `value`)
    torch.cuda.synchronize()
    time.sleep(0.5)
    for _ in range(args.warmup):
        pipe.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        pipe.step()
    torch.cuda.synchronize()
    ms_from_idle = (time.perf_counter() - t0) * 1e3 / max(args.steps, 1)
    ms, phases = time_steps(pipe, torch, args.steps, args.warmup)
    work = algorithmic_work(w, B)

    # dominant kernel = the phase that takes the most time
    norm_ms, clip_ms, grad_ms, noise_ms = phases
    nlayers = len(w.layers)
    if grad_ms >= norm_ms:
        flops, byts, dur_ms, kname = work["gemm_flops"], work["gemm_bytes"], grad_ms, "clipped-sum GEMMs of all layers with their split-K folds (and the noise that the folds add, where the configuration has noise); aligned 16-bit / 8-bit layers share one GEMM launch"
    else:
        flops, byts, dur_ms, kname = work["norm_flops"], work["norm_bytes"], norm_ms, "squared-norm kernel (dp_layer_sqnorm)"
    peak_tf = PEAK_MFMA_TFLOPS[w.dtype]
    ai = flops / max(byts, 1)
    if ai >= peak_tf * 1e12 / (PEAK_HBM_GBS * 1e9):
        ach = flops / (dur_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": ach, "peak": peak_tf, "unit": "TFLOP/s", "frac": ach / peak_tf}
    else:
        ach = byts / (dur_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS}
    traffic = MEASURED_TRAFFIC.get(w.name) if (args.batch is None and args.path == "auto" and args.dtype is None) else None
    # achieved / traffic are per step: the phase of the dominant kernel (for the transformer configuration one GEMM
    # launch for the four layers and a fold per layer), timed with HIP events inside the timed steps
    roof.update({"traffic": traffic, "kernel": kname, "layers_per_step": nlayers,
                 "phase_ms": dur_ms,
                 "algorithmic_flops_per_step": flops, "algorithmic_bytes_per_step": byts})

    phases_out = {
        "sqnorm_ms": norm_ms, "clip_ms": clip_ms, "clipped_grad_ms": grad_ms, "noise_ms": noise_ms,
        "sqnorm_tflops": work["norm_flops"] / (norm_ms * 1e-3) / 1e12,
        "sqnorm_gbs": work["norm_bytes"] / (norm_ms * 1e-3) / 1e9,
        "clipped_grad_tflops": work["gemm_flops"] / (grad_ms * 1e-3) / 1e12,
        "clipped_grad_gbs": work["gemm_bytes"] / (grad_ms * 1e-3) / 1e9,
    }
    noise_fused = w.noise_std > 0
    if noise_fused:
        # the noise is added inside the clipped-sum phase (by the kernels that fold the K slices): no pass of its own
        phases_out["noise_ms"] = 0.0
        phases_out["noise"] = "added by the split-K reduce kernels, inside clipped_grad_ms"
    elif noise_ms > 0 and work["noise_bytes"]:
        phases_out["noise_gbs"] = work["noise_bytes"] / (noise_ms * 1e-3) / 1e9

    # bias parameters (the first of the "next" rows): per-example bias gradients + their squared norms for every
    # layer, then the clipped bias sums; timed on their own, not part of `value`
    es = 2 if w.dtype in ("bf16", "f16") else (1 if w.dtype.startswith("f8") else 4)
    rows = [torch.empty((B, spec.d_out), dtype=torch.float32, device="cuda") for spec in w.layers]
    gbs = [torch.empty(spec.d_out, dtype=torch.float32, device="cuda") for spec in w.layers]
    evb = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    tb = np.zeros(2)
    for rep in range(5 + 2):
        evb[0].record()
        for (A, G), u in zip(pipe.dev, rows):
            dp.bias_sqnorm(G, pipe.s, u, accumulate=True)
        evb[1].record()
        for u, gb in zip(rows, gbs):
            dp.clipped_bias_grad(u, pipe.c, gb)
        evb[2].record()
        torch.cuda.synchronize()
        if rep >= 2:
            tb += [evb[0].elapsed_time(evb[1]), evb[1].elapsed_time(evb[2])]
    tb /= 5
    bias_bytes = sum(B * spec.T * spec.d_out * es + 4 * B * spec.d_out for spec in w.layers)
    bias_out = {"bias_sqnorm_ms": tb[0], "clipped_bias_grad_ms": tb[1], "bias_sqnorm_gbs": bias_bytes / (tb[0] * 1e-3) / 1e9,
                "algorithmic_bytes": bias_bytes}
    if len(w.layers) > 1:
        # the same bias rows and norms taken inside the several-layers norm call (by the Gram kernel where the
        # layers share its launch): the norm phase with and without them
        d_wb = dp.layer_descs(pipe.dev, bias_rows=rows)
        ws_wb = torch.empty(max(16, dp.layers_workspace_bytes(d_wb[0], B, d_wb[2], args.path)), dtype=torch.uint8, device="cuda")
        tf = np.zeros(2)
        for rep in range(10 + 3):
            evb[0].record()
            dp.layers_sqnorm(pipe.dev, pipe.s, path=args.path, workspace=ws_wb, descs=d_wb, C=w.C, clip=pipe.c)
            evb[1].record()
            dp.layers_sqnorm(pipe.dev, pipe.s, path=args.path, workspace=pipe.ws_layers, descs=pipe.descs, C=w.C, clip=pipe.c)
            evb[2].record()
            torch.cuda.synchronize()
            if rep >= 3:
                tf += [evb[0].elapsed_time(evb[1]), evb[1].elapsed_time(evb[2])]
        tf /= 10
        bias_out["sqnorm_with_bias_rows_ms"] = tf[0]
        bias_out["sqnorm_without_ms"] = tf[1]
        del ws_wb
    del rows, gbs
    # LayerNorm scale and shift rows (Algorithm 5) of a layer of the first layer's input width: G and the normalised
    # input of the same shape, read once each (the first layer's A and a same-shaped slice of values stand in)
    A0 = pipe.dev[0][0]
    if A0.dim() == 3:
        H0 = torch.roll(A0.view(torch.uint8) if w.dtype.startswith("f8") else A0, 1, 0)
        H0 = H0.view(A0.dtype) if w.dtype.startswith("f8") else H0
        tl = 0.0
        for rep in range(5 + 2):
            evb[0].record()
            dp.layernorm_sqnorm(H0, A0, pipe.s, accumulate=True)
            evb[1].record()
            torch.cuda.synchronize()
            if rep >= 2:
                tl += evb[0].elapsed_time(evb[1])
        tl /= 5
        ln_bytes = 2 * A0.numel() * A0.element_size() + 2 * 4 * A0.shape[0] * A0.shape[2]
        bias_out["layernorm_sqnorm_ms"] = tl
        bias_out["layernorm_sqnorm_gbs"] = ln_bytes / (tl * 1e-3) / 1e9
        bias_out["layernorm_shape"] = [int(x) for x in A0.shape]
        del H0

    if not args.no_others and args.batch is None and not w.dtype.startswith("f8"):
        # the row kernels at sizes where their launches no longer count: one layer's G of the widest and of the
        # narrowest output (and a G / Hbar pair for the LayerNorm rows) at the configuration's batch and at four times
        # it, cold (a 512 MB buffer is read in between), values drawn on the device (the timing does not depend on them)
        tdt = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[w.dtype]
        fl = torch.zeros(1 << 27, dtype=torch.float32, device="cuda")
        Tm = max(spec.T for spec in w.layers)
        sweep = {}
        for d in sorted({max(spec.d_out for spec in w.layers), min(spec.d_out for spec in w.layers)}):
            for mult in (1, 4):
                Bs = B * mult
                Gs = torch.randn((Bs, Tm, d), device="cuda", dtype=torch.float32).to(tdt)
                Hs = torch.randn((Bs, Tm, d), device="cuda", dtype=torch.float32).to(tdt)
                ss = torch.zeros(Bs, device="cuda")
                us = torch.empty((Bs, d), device="cuda")
                tt = np.zeros(2)
                for rep in range(2 + 5):
                    fl.max()
                    evb[0].record()
                    dp.bias_sqnorm(Gs, ss, us)
                    evb[1].record()
                    fl.max()
                    torch.cuda.synchronize()
                    t_b = evb[0].elapsed_time(evb[1])
                    evb[0].record()
                    dp.layernorm_sqnorm(Gs, Hs, ss)
                    evb[1].record()
                    torch.cuda.synchronize()
                    if rep >= 2:
                        tt += [t_b, evb[0].elapsed_time(evb[1])]
                tt /= 5
                nb = Gs.numel() * Gs.element_size()
                sweep[f"B={Bs},T={Tm},d={d}"] = {
                    "bias_sqnorm_ms": tt[0], "bias_sqnorm_gbs": (nb + 4 * Bs * d) / (tt[0] * 1e-3) / 1e9,
                    "bias_sqnorm_hbm_frac": (nb + 4 * Bs * d) / (tt[0] * 1e-3) / 1e9 / PEAK_HBM_GBS,
                    "layernorm_sqnorm_ms": tt[1], "layernorm_sqnorm_gbs": (2 * nb + 8 * Bs * d) / (tt[1] * 1e-3) / 1e9,
                    "layernorm_sqnorm_hbm_frac": (2 * nb + 8 * Bs * d) / (tt[1] * 1e-3) / 1e9 / PEAK_HBM_GBS,
                    "input_mb": nb / 1e6}
                del Gs, Hs, ss, us
        bias_out["sweep_cold"] = sweep
        del fl

    others = {}
    if not args.no_others and args.batch is None:
        flush = torch.zeros(1 << 27, dtype=torch.float32, device="cuda")
        for name in wl.WORKLOADS:
            if name == args.workload:
                continue
            w2, l2 = wl.generate(name)
            p2 = Pipeline(w2, l2, torch, dp, "auto")
            ms2, ph2 = time_steps(p2, torch, 50, 5)
            wk2 = algorithmic_work(w2, p2.B)
            others[name] = {"examples_per_s": p2.B / (ms2 * 1e-3), "ms_per_step": ms2,
                            "sqnorm_ms": ph2[0], "clipped_grad_ms": ph2[2],
                            "sqnorm_gbs": wk2["norm_bytes"] / (ph2[0] * 1e-3) / 1e9,
                            "sqnorm_tflops": wk2["norm_flops"] / (ph2[0] * 1e-3) / 1e12,
                            "clipped_grad_tflops": wk2["gemm_flops"] / (ph2[2] * 1e-3) / 1e12,
                            "clipped_grad_gbs": wk2["gemm_bytes"] / (ph2[2] * 1e-3) / 1e9}
            # the same step captured once into a HIP graph and replayed (the library neither allocates nor
            # synchronises, so a step is capturable): takes the host's launch rate out of the small configurations
            # once as a graph of one step and once as a graph of 16 steps: a replay costs the runtime about 10 us
            # whatever the graph holds, which a one-step graph of a 10-20 us step cannot win back
            for n_in_graph, key in ((1, "ms_per_step_graph"), (16, "ms_per_step_graph_of_16_steps")):
                try:
                    side = torch.cuda.Stream()
                    graph = torch.cuda.CUDAGraph()
                    with torch.cuda.stream(side):
                        p2.step()
                        side.synchronize()
                        with torch.cuda.graph(graph, stream=side):
                            for _ in range(n_in_graph):
                                p2.step()
                    torch.cuda.synchronize()
                    for _ in range(5):
                        graph.replay()
                    torch.cuda.synchronize()
                    reps = max(4, 64 // n_in_graph)
                    t0 = time.perf_counter()
                    for _ in range(reps):
                        graph.replay()
                    torch.cuda.synchronize()
                    others[name][key] = (time.perf_counter() - t0) * 1e3 / (reps * n_in_graph)
                    del graph
                except Exception as exc:          # reported, never fatal for the benchmark line
                    others[name][key] = None
                    others[name]["graph_error"] = str(exc)[:200]
            # the same with cold caches (the timings above are back-to-back steps over inputs that fit the caches)
            pc = time_steps_cold(p2, torch, 10, flush)
            others[name]["cold"] = {"sqnorm_ms": pc[0], "clipped_grad_ms": pc[2],
                                    "sqnorm_gbs": wk2["norm_bytes"] / (pc[0] * 1e-3) / 1e9,
                                    "clipped_grad_gbs": wk2["gemm_bytes"] / (pc[2] * 1e-3) / 1e9}
            del p2, l2
            if name in ("dense", "mlp", "rnn"):
                # the same per-example shapes at many times the batch (up to 200 - 600 MB of inputs), cold: at the
                # configuration's own size the step is a few launches of a few microseconds, here the kernels have
                # bytes to move
                sweep = {}
                for mult in {"dense": (256, 4096, 16384), "mlp": (16, 64, 256), "rnn": (16, 64)}[name]:
                    ws_, ls_ = wl.generate(name, B=w2.B * mult)
                    ps_ = Pipeline(ws_, ls_, torch, dp, "auto")
                    del ls_
                    for _ in range(2):
                        ps_.step()
                    pcs = time_steps_cold(ps_, torch, 6, flush)
                    wks = algorithmic_work(ws_, ps_.B)
                    sweep[f"B={ps_.B}"] = {
                        "sqnorm_ms": pcs[0], "clipped_grad_ms": pcs[2],
                        "sqnorm_gbs": wks["norm_bytes"] / (pcs[0] * 1e-3) / 1e9,
                        "sqnorm_hbm_frac": wks["norm_bytes"] / (pcs[0] * 1e-3) / 1e9 / PEAK_HBM_GBS,
                        "clipped_grad_gbs": wks["gemm_bytes"] / (pcs[2] * 1e-3) / 1e9,
                        "clipped_grad_tflops": wks["gemm_flops"] / (pcs[2] * 1e-3) / 1e12,
                        "input_mb": wks["norm_bytes"] / 1e6}
                    del ps_
                others[name]["sweep_cold"] = sweep
        # the transformer configuration with fp16 inputs (G and C carry a loss scale of 1024): the same kernels with
        # the fp16 matrix instruction
        w16, l16 = wl.generate("transformer", dtype="f16", g_scale=1024.0)
        w16 = dataclasses.replace(w16, dtype="f16", C=w16.C * 1024.0, noise_std=w16.noise_std * 1024.0)
        p16 = Pipeline(w16, l16, torch, dp, "auto")
        ms16, ph16 = time_steps(p16, torch, 20, 3)
        wk16 = algorithmic_work(w16, p16.B)
        others["transformer_f16"] = {"examples_per_s": p16.B / (ms16 * 1e-3), "ms_per_step": ms16,
                                     "sqnorm_ms": ph16[0], "clipped_grad_ms": ph16[2],
                                     "sqnorm_tflops": wk16["norm_flops"] / (ph16[0] * 1e-3) / 1e12,
                                     "clipped_grad_tflops": wk16["gemm_flops"] / (ph16[2] * 1e-3) / 1e12}
        del p16, l16
        # per-layer clipping (threshold C / sqrt(m) per layer): every layer names its own norm and clip arrays in the
        # same two calls; the Gram launch stays shared
        wp, lp = wl.generate("transformer")
        pp = Pipeline(wp, lp, torch, dp, "auto")
        m = len(pp.dev)
        sq_l = [torch.zeros(pp.B, dtype=torch.float32, device="cuda") for _ in range(m)]
        cl_l = [torch.zeros(pp.B, dtype=torch.float32, device="cuda") for _ in range(m)]
        Cl = wp.C / math.sqrt(m)
        pp.descs = dp.layer_descs(pp.dev, groups=[(sq_l[l], cl_l[l], Cl) for l in range(m)])
        order = sorted(range(m), key=lambda li: pp.dev[li][0].shape[2] + pp.dev[li][1].shape[2])
        sizes = [spec.d_in * spec.d_out for spec in wp.layers]
        starts = np.concatenate([[0], np.cumsum(sizes)]).tolist()
        pp.descs_cg = dp.layer_descs(pp.dev_cg, [pp.grads[li] for li in order], [starts[li] for li in order],
                                     groups=[(sq_l[li], cl_l[li], Cl) for li in order])
        msp, php = time_steps(pp, torch, 20, 3)
        others["transformer_per_layer_clipping"] = {"examples_per_s": pp.B / (msp * 1e-3), "ms_per_step": msp,
                                                    "sqnorm_ms": php[0], "clipped_grad_ms": php[2],
                                                    "threshold_per_layer": Cl}
        del pp, lp, sq_l, cl_l
        # ... and with 8-bit inputs, activations e4m3 and backpropagated gradients e5m2: the 64-deep 8-bit matrix
        # instruction, twice the rate for half the bytes
        w8, l8 = wl.generate("transformer", dtype="f8")
        w8 = dataclasses.replace(w8, dtype="f8")
        p8 = Pipeline(w8, l8, torch, dp, "auto")
        ms8, ph8 = time_steps(p8, torch, 20, 3)
        wk8 = algorithmic_work(w8, p8.B)
        others["transformer_f8"] = {"examples_per_s": p8.B / (ms8 * 1e-3), "ms_per_step": ms8, "storage": "A e4m3, G e5m2",
                                    "sqnorm_ms": ph8[0], "clipped_grad_ms": ph8[2],
                                    "sqnorm_tflops": wk8["norm_flops"] / (ph8[0] * 1e-3) / 1e12,
                                    "clipped_grad_tflops": wk8["gemm_flops"] / (ph8[2] * 1e-3) / 1e12}
        del p8, l8
        # the convolution configuration again, given by its input image (implicit unfolding: 16.8 MB of X instead of
        # the 151 MB patch matrix); same flops, same outputs as "conv"
        spec, Xn, Gn = wl.generate_conv_image()
        Xd, Gd = to_dev(Xn, torch), to_dev(Gn, torch)
        del Xn, Gn
        Bc, KH, KW, pad = spec["B"], spec["KH"], spec["KW"], spec["pad"]
        d_in, d_out = KH * KW * spec["C"], spec["d_out"]
        T = (spec["H"] + 2 * pad - KH + 1) * (spec["W"] + 2 * pad - KW + 1)
        geo = (Bc, spec["H"], spec["W"], spec["C"], KH, KW, pad, d_out, dp.DP_BF16)
        ws1 = torch.empty(dp.conv_workspace_bytes(dp.DP_OP_SQNORM, *geo), dtype=torch.uint8, device="cuda")
        ws2 = torch.empty(dp.conv_workspace_bytes(dp.DP_OP_CLIPPED_GRAD, *geo), dtype=torch.uint8, device="cuda")
        sc, cc = torch.zeros(Bc, device="cuda"), torch.zeros(Bc, device="cuda")
        gc = torch.zeros((d_in, d_out), device="cuda")

        def conv_step(ev=None):
            if ev:
                ev[0].record()
            dp.conv_sqnorm(Xd, Gd, KH, KW, pad, sc, workspace=ws1)
            if ev:
                ev[1].record()
            dp.clip_factors(sc, spec["C_clip"], cc)
            dp.conv_clipped_grad(Xd, Gd, cc, KH, KW, pad, gc, workspace=ws2)
            if ev:
                ev[2].record()

        res = {}
        for mode in ("warm", "cold"):
            n = 50 if mode == "warm" else 10
            for _ in range(3):
                conv_step()
            evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n)]
            for k in range(n):
                if mode == "cold":
                    flush.max()
                conv_step(evs[k])
            torch.cuda.synchronize()
            a = sum(e[0].elapsed_time(e[1]) for e in evs) / n
            b = sum(e[1].elapsed_time(e[2]) for e in evs) / n
            res[mode] = {"sqnorm_ms": a, "clip_and_clipped_grad_ms": b,
                         "sqnorm_tflops": 2.0 * Bc * T * d_in * d_out / (a * 1e-3) / 1e12,
                         "clipped_grad_tflops": 2.0 * Bc * T * d_in * d_out / (b * 1e-3) / 1e12}
        res["input_bytes"] = int(Xd.numel() * 2 + Gd.numel() * 2)
        others["conv_from_image"] = res
        del flush, Xd, Gd
        # Stacks of unfolded convolutions shaped like the paper's image models (Section 6: ResNet / VGG at 20-32 examples):
        # every layer's norms, the clip factors and the clipped sums with noise through dp_layers_step, bf16.
        # (positions, patch columns, channels) per layer; N(0, 1) inputs drawn on the device.
        stacks = {
            "resnet18_like_32x32_B32": (32, [(1024, 27, 64)] + [(1024, 576, 64)] * 4 + [(256, 576, 128)] + [(256, 1152, 128)] * 3
                                        + [(64, 1152, 256)] + [(64, 2304, 256)] * 3 + [(16, 2304, 512)] + [(16, 4608, 512)] * 3 + [(1, 512, 10)]),
            "resnet18_like_256x256_B20": (20, [(16384, 147, 64)] + [(4096, 576, 64)] * 4 + [(1024, 576, 128), (1024, 64, 128)]
                                          + [(1024, 1152, 128)] * 3 + [(256, 1152, 256), (256, 128, 256)] + [(256, 2304, 256)] * 3
                                          + [(64, 2304, 512), (64, 256, 512)] + [(64, 4608, 512)] * 3 + [(1, 512, 10)]),
        }
        stack_out = {}
        for sname, (Bs, shapes) in stacks.items():
            gen = torch.Generator(device="cuda").manual_seed(wl.BASE_SEED + 77)
            lay = []
            for (T, di, do) in shapes:
                shp_a, shp_g = ((Bs, T, di), (Bs, T, do)) if T > 1 else ((Bs, di), (Bs, do))
                lay.append((torch.randn(shp_a, device="cuda", generator=gen).to(torch.bfloat16),
                            torch.randn(shp_g, device="cuda", generator=gen).to(torch.bfloat16)))
            sizes = [di * do for (_, di, do) in shapes]
            starts = np.concatenate([[0], np.cumsum(sizes)]).tolist()
            flat = torch.zeros(int(sum(sizes)), device="cuda")
            grads = [flat[starts[i]:starts[i + 1]].view(di, do) for i, (_, di, do) in enumerate(shapes)]
            descs = dp.layer_descs(lay, grads, starts[:-1])
            arr, _, dtc = descs
            wss = torch.empty(max(16, dp.layers_workspace_bytes(arr, Bs, dtc, "auto"), dp.layers_clipped_workspace_bytes(arr, Bs, dtc)),
                              dtype=torch.uint8, device="cuda")
            sq, cl = torch.zeros(Bs, device="cuda"), torch.zeros(Bs, device="cuda")
            for _ in range(3):
                dp.layers_step(descs, 1.0, sq, cl, wss, noise_std=1.0, seed=1)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(20):
                dp.layers_step(descs, 1.0, sq, cl, wss, noise_std=1.0, seed=1)
            torch.cuda.synchronize()
            mss = (time.perf_counter() - t0) / 20 * 1e3
            in_bytes = sum(Bs * T * (di + do) * 2 for (T, di, do) in shapes)
            stack_out[sname] = {"layers": len(shapes), "examples_per_s": Bs / (mss * 1e-3), "ms_per_step": mss,
                                "input_mb": in_bytes / 1e6, "clipped_sum_gflop": sum(2.0 * Bs * T * di * do for (T, di, do) in shapes) / 1e9}
            del lay, grads, flat, wss
        others["image_model_stacks"] = stack_out

    out = {
        "metric": "examples/sec for norm+clip+clipped-sum per layer",
        "value": B / (ms * 1e-3), "unit": "examples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: B={B}, " + ", ".join(f"{s.name} T={s.T} {s.d_in}->{s.d_out}" for s in w.layers)
                   + f", C={w.C}" + (f", noise std={w.noise_std}" if w.noise_std > 0 else "")
                   + (f", inputs stored as {args.dtype}" if args.dtype else ""),
                   "path": args.path, "parallelism": "single GPU", "untimed_spinup_s": SPINUP_S},
        "roofline": roof, "phases": phases_out, "bias_terms": bias_out, "other_workloads": others,
    }
    out["ms_per_step_from_idle"] = ms_from_idle
    if not args.no_peaks:
        peaks = measured_peaks(torch, dp)
        out["measured_peaks"] = peaks
        if roof["bound"] == "mfma":
            key = {"bf16": "bf16", "f16": "f16"}.get(w.dtype, "f8_e4m3_e5m2" if w.dtype.startswith("f8") else None)
            if key is not None:
                roof["peak_measured"] = peaks[f"mfma_{key}_random_operands_tflops"]
                roof["frac_of_measured"] = roof["achieved"] / roof["peak_measured"]
        else:
            roof["peak_measured"] = peaks["hbm_read_gbs"]
            roof["frac_of_measured"] = roof["achieved"] / roof["peak_measured"]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w.name, min(w.B, B))
        if not args.no_others and args.batch is None:
            # the oracle on every other configuration (all host threads; one thread too for the three small ones)
            for name in wl.WORKLOADS:
                if name == w.name or name not in others:
                    continue
                sample = min(wl.WORKLOADS[name].B, 16) if name == "conv" else wl.WORKLOADS[name].B
                others[name]["cpu_baseline"] = cpu_baseline(name, sample)
                if name in ("dense", "mlp", "rnn"):
                    others[name]["cpu_baseline_1_thread"] = cpu_baseline(name, sample, threads=1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
