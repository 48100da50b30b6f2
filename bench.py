#!/usr/bin/env python3
"""Benchmark of the SMILE bi-level MoE layer forward on one MI355X.

One "step" is one pass of the whole hot path over one batch of seeded synthetic tokens: gate logits -> bi-level
routing with capacity -> dispatch -> expert FFN (up, down) -> combine -> load-balancing loss, all through the
C-ABI library (smile_layer_forward without expert buffers: the permutations are fused into the expert GEMMs),
inputs and weights resident in HBM.

Default run (--workload all): the headline is the largest configuration, cfg5 (T=65536, d=1024, F=4096, 32 x 8
experts, skewed router); cfg1 .. cfg4 are timed the same way in the same process and reported under "configs" of
the same JSON line.  For every configuration:
  * the timed region is exactly K calls bracketed by synchronisation (`ms_per_step`, `value`), with one HIP event
    per step boundary on the stream (`ms_per_step_event_median`) and a HIP event pair that the library attaches to
    the launch of the dominant kernel, the up-projection grouped GEMM, so that `roofline` comes from that kernel's
    own duration inside the timed region;
  * a second, instrumented pass attaches an event pair to EVERY kernel of the step (smile_kernel_timing) and to the
    stand-alone dispatch / combine kernels: `kernels_us`, `hbm` and the launch-gap sum come from those
    kernel-own durations, not from intervals that include launch latency.
`roofline.bound` is the binding one of the two lower bounds of the up-projection: 2*K*d*F flop at the bf16 MFMA
peak against its compulsory bytes (all expert weights once + kept rows in + hidden rows out) at the HBM peak;
both fractions are always given.  The headline also gets a training leg (forward that saves activations +
backward) and the CPU oracle timed on the host cores.  Prints ONE JSON line.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 / fp16 MFMA (published)
PEAK_F32_TFLOPS = 157.3       # MI355X fp32 vector (published)
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E (published)
# What the chip delivered to the microbenchmark paper_2212_05191_amd/peaks_probe (profiles/mi355x_measured_peaks.txt):
# read-only streaming of expert-weight tiles through direct-to-LDS loads, and back-to-back MFMAs without loads.
MEASURED_HBM_GBS = 6100.0
MEASURED_BF16_TFLOPS = 2485.0

# HBM bytes per launch of the up-projection GEMM from rocprofv3 --pmc passes (FETCH_SIZE, then WRITE_SIZE, each
# scaled by what the same counter reads for a plain device copy of known size); the summary that backs each
# figure is named beside it.  Workloads without a tracked summary report null.
MEASURED_TRAFFIC = {
    "cfg2": (137.38e6, "profiles/bench_cfg2_hbm_traffic_pmc.txt"),
    "cfg3": (738.33e6, "profiles/bench_cfg3_hbm_traffic_pmc.txt"),
    "cfg4": (840.35e6, "profiles/bench_cfg4_hbm_traffic_pmc.txt"),
    "cfg5": (2262.06e6, "profiles/bench_cfg5_hbm_traffic_pmc.txt"),
}

PRE_WARM_S = 0.25   # untimed ramp before the warm-up steps of every configuration
HEADLINE = "cfg5"
ALL_CONFIGS = ["cfg5", "cfg1", "cfg2", "cfg3", "cfg4"]


class Hip:
    """The few HIP runtime calls the benchmark needs itself (events on the library's stream)."""

    def __init__(self):
        self.lib = ctypes.CDLL("libamdhip64.so")
        self.lib.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.lib.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.lib.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def event(self):
        e = ctypes.c_void_p()
        assert self.lib.hipEventCreate(ctypes.byref(e)) == 0
        return e

    def record(self, e, stream):
        assert self.lib.hipEventRecord(e, ctypes.c_void_p(stream)) == 0

    def ms(self, a, z):
        out = ctypes.c_float()
        assert self.lib.hipEventElapsedTime(ctypes.byref(out), a, z) == 0
        return float(out.value)

    def destroy(self, events):
        for e in events:
            self.lib.hipEventDestroy(e)


def kernel_label(name: str) -> str:
    """Short label of a kernel name as the library reports it (template arguments and parentheses dropped)."""
    return name.strip("()").split("<")[0]


def timed_kernels(hip, lib, ctx_handle, call, reps, max_kernels=12):
    """Median kernel-own durations (us) of every kernel `call` launches: list of (label, us) in launch order."""
    import numpy as np
    import torch
    arrays, per_rep = [], []
    for _ in range(reps):
        evs = [hip.event() for _ in range(2 * max_kernels)]
        arr = (ctypes.c_void_p * (2 * max_kernels))(*[e.value for e in evs])
        arrays.append((evs, arr))
    labels = None
    for evs, arr in arrays:
        assert lib.smile_kernel_timing(ctx_handle, arr, max_kernels) == 0
        call()
        n = lib.smile_kernel_timing_count(ctx_handle)
        if labels is None:
            labels = [kernel_label(lib.smile_kernel_timing_name(ctx_handle, i).decode()) for i in range(n)]
        per_rep.append(n)
    assert lib.smile_kernel_timing(ctx_handle, None, 0) == 0
    torch.cuda.synchronize()
    us = []
    for i in range(len(labels)):
        us.append(1e3 * float(np.median([hip.ms(evs[2 * i], evs[2 * i + 1]) for (evs, _), n in zip(arrays, per_rep) if i < n])))
    for evs, _ in arrays:
        hip.destroy(evs)
    return list(zip(labels, us))


def bench_config(name, steps, warmup, hip, with_training, with_cpu, copy_calibration=False):
    import numpy as np
    import torch
    from paper_2212_05191_amd import binding as B
    from paper_2212_05191_amd import workloads as wl
    from paper_2212_05191_amd.runner import GpuLayer

    lib = B.load()
    cfg = wl.get_config(name)
    layer = GpuLayer(cfg, workers=16)
    b, h = layer.buf, layer.ctx.handle
    stream = torch.cuda.current_stream().cuda_stream
    p = B._ptr
    io = layer.io_fused     # no expert buffers: dispatch / combine fused into the expert GEMMs

    def step(ev=None):
        io.prof_up_start, io.prof_up_stop = (ev[0], ev[1]) if ev is not None else (None, None)
        st = lib.smile_layer_forward(h, ctypes.byref(io), stream)
        if st != 0:
            raise B.SmileError(st, "smile_layer_forward")

    # clock and cache ramp, untimed: after the host-side set-up (seconds of idle GPU) the first tens of
    # milliseconds of work run slower than the steady state; then the W warm-up steps proper
    c0, pre_warm_steps = time.perf_counter(), 0
    while time.perf_counter() - c0 < PRE_WARM_S:
        for _ in range(8):
            step()
        pre_warm_steps += 8
        torch.cuda.synchronize()
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps; an event at every step boundary and a pair around the dominant kernel
    pairs = [(hip.event(), hip.event()) for _ in range(steps)]
    marks = [hip.event() for _ in range(steps + 1)]
    for e in marks:   # first use of an event outside the timed region (whatever the runtime sets up lazily)
        hip.record(e, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    hip.record(marks[0], stream)
    for k in range(steps):
        step(pairs[k])
        hip.record(marks[k + 1], stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    sec_per_step = (t1 - t0) / steps
    step_ms_events = [hip.ms(marks[k], marks[k + 1]) for k in range(steps)]
    dom_ms = float(np.mean([hip.ms(a, z) for a, z in pairs]))
    hip.destroy([e for pr in pairs for e in pr] + marks)
    io.prof_up_start = io.prof_up_stop = None

    if copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    kept = int(b.kept_count.sum().item())
    ecnt = b.expert_count.cpu().numpy()
    half = cfg.dtype != "f32"
    s = 2 if half else 4
    d, F, T, N, n, m = cfg.d_model, cfg.d_ff, cfg.T, cfg.N, cfg.n_groups, cfg.m_local
    up_flops = 2.0 * kept * d * F
    up_bytes = N * d * F * s + kept * d * s + kept * F * s

    # ---- instrumented pass (not part of `value`): an event pair on every kernel of the fused step, then on the
    # stand-alone dispatch / combine kernels of the materialised path
    reps = max(5, min(steps, 20))
    fused = timed_kernels(hip, lib, h, step, reps)
    kernels_us = {}
    gemms = [i for i, (lbl, _) in enumerate(fused) if lbl.startswith("grouped_gemm_nt")]
    for i, (lbl, us) in enumerate(fused):
        key = lbl
        if gemms and i == gemms[0]:
            key = "expert_ffn_up"
        elif gemms and i == gemms[-1]:
            key = "expert_ffn_down"
        kernels_us[key] = round(kernels_us.get(key, 0.0) + us, 2)
    kernel_sum_us = sum(us for _, us in fused)

    def separate():
        st = lib.smile_dispatch(h, p(layer.x), p(b.group_idx), p(b.local_idx), p(b.slot), p(b.xe), stream)
        assert st == 0
    disp = timed_kernels(hip, lib, h, separate, reps)

    def separate2():
        st = lib.smile_combine(h, p(b.xe), p(b.group_idx), p(b.local_idx), p(b.slot), p(b.gate), p(b.y), stream)
        assert st == 0
    # combine reads the expert buffer it is given: xe (just dispatched, same shape and dtype as ye) serves as input
    comb = timed_kernels(hip, lib, h, separate2, reps)
    gate_us = sum(us for lbl, us in fused if lbl.startswith("gate_logits")) or None   # wide routers: several passes
    route_us = sum(us for lbl, us in fused if lbl.startswith("route_") or lbl.startswith("finalize_map"))
    up_us, down_us = kernels_us.get("expert_ffn_up"), kernels_us.get("expert_ffn_down")
    alg_bytes = {
        "gate_logits": (T * d * s + (n + m) * d * s + 4 * T * (n + m), gate_us),
        "dispatch": (2 * kept * d * s + 12 * T, disp[0][1]),
        "combine": (kept * d * s + T * d * s + 16 * T, comb[0][1]),
        "expert_ffn_up": (up_bytes, up_us),
        "expert_ffn_down": (N * d * F * s + kept * F * s + kept * d * s, down_us),
    }
    hbm = {}
    for k, (nbytes, us) in alg_bytes.items():
        if us:
            gbs = nbytes / (us * 1e-6) / 1e9
            hbm[k] = {"kernel_us": round(us, 2), "alg_MB": round(nbytes / 1e6, 2), "GBps": round(gbs, 1),
                      "frac_of_8TBps": round(gbs / PEAK_HBM_GBS, 4),
                      "frac_of_measured_peak": round(gbs / MEASURED_HBM_GBS, 4)}

    # ---- roofline of the dominant kernel, from its event pairs inside the timed region
    dom_s = dom_ms * 1e-3
    if half:
        achieved_tflops = up_flops / dom_s / 1e12
        achieved_gbs = up_bytes / dom_s / 1e9
        t_mfma, t_hbm = up_flops / (PEAK_BF16_TFLOPS * 1e12), up_bytes / (PEAK_HBM_GBS * 1e9)
        traffic, traffic_src = MEASURED_TRAFFIC.get(cfg.name, (None, None))
        common = {"kernel": "grouped_gemm_nt_kernel (expert FFN up-projection + activation)",
                  "avg_launch_us": round(dom_ms * 1e3, 2), "alg_flops_per_launch": up_flops,
                  "alg_bytes_per_launch": up_bytes,
                  "lower_bound_us": {"mfma": round(t_mfma * 1e6, 2), "hbm": round(t_hbm * 1e6, 2)},
                  "frac_mfma": round(achieved_tflops / PEAK_BF16_TFLOPS, 4),
                  "frac_hbm": round(achieved_gbs / PEAK_HBM_GBS, 4),
                  "traffic": traffic, "traffic_source": traffic_src}
        if t_hbm >= t_mfma:
            roofline = {"bound": "hbm", "achieved": round(achieved_gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": round(achieved_gbs / PEAK_HBM_GBS, 4),
                        "frac_of_measured_peak": round(achieved_gbs / MEASURED_HBM_GBS, 4), **common}
        else:
            roofline = {"bound": "mfma", "achieved": round(achieved_tflops, 2), "peak": PEAK_BF16_TFLOPS,
                        "unit": "TFLOP/s", "frac": round(achieved_tflops / PEAK_BF16_TFLOPS, 4),
                        "frac_of_measured_peak": round(achieved_tflops / MEASURED_BF16_TFLOPS, 4), **common}
    else:
        achieved_tflops = up_flops / dom_s / 1e12
        roofline = {"bound": "alu", "kernel": "grouped_gemm_nt_f32_kernel (fp32 FMA path of the tiny configuration)",
                    "achieved": round(achieved_tflops, 3), "peak": PEAK_F32_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(achieved_tflops / PEAK_F32_TFLOPS, 5), "traffic": None,
                    "avg_launch_us": round(dom_ms * 1e3, 2), "alg_flops_per_launch": up_flops}

    out = {
        "workload": f"{cfg.name}: T={T} d_model={d} d_ff={F} experts={n}x{m} capacity={cfg.capacity} "
                    f"(cf {cfg.capacity_factor}) {cfg.dtype} {cfg.act}" + (" skewed router" if cfg.skew else ""),
        "tokens_per_s": round(T / sec_per_step, 1),
        "ms_per_step": round(sec_per_step * 1e3, 4),
        "ms_per_step_event_median": round(float(np.median(step_ms_events)), 4),
        "steps": steps, "pre_warm_steps": pre_warm_steps,
        "T": T, "kept_tokens": kept, "dropped_tokens": T - kept,
        "max_over_mean_expert_load": round(float(ecnt.max() / max(ecnt.mean(), 1e-9)), 3),
        "roofline": roofline,
        "expert_gemm_mfma_frac": (round(2 * up_flops / ((up_us + down_us) * 1e-6) / 1e12 / PEAK_BF16_TFLOPS, 4)
                                  if half and up_us and down_us else None),
        "kernels_us": kernels_us,
        "route_kernels_us": round(route_us, 2),
        "launches_per_step": len(fused),
        # event-timed step minus the sum of the kernel-own durations of the instrumented pass (launch gaps; the
        # instrumented kernels run a little slower than in the timed region, so this can come out negative)
        "step_minus_kernel_sum_us": round(float(np.median(step_ms_events)) * 1e3 - kernel_sum_us, 2),
        "hbm": hbm,
    }

    # ---- training step = forward with expert buffers and saved activations, then the backward pass, each
    # through its single chained entry point (not part of `value`)
    if with_training:
        layer.enable_saved_activations()
        layer.prepare_backward(wl.gen_output_grad(cfg))
        bws = layer.bwd_workspace
        bw_bytes = bws.numel()

        def fwd_train():
            st = lib.smile_layer_forward(h, ctypes.byref(layer.io), stream)
            if st != 0:
                raise B.SmileError(st, "smile_layer_forward")

        def bwd():
            st = lib.smile_layer_backward(h, ctypes.byref(layer.bwd_io), ctypes.c_float(1.0), p(bws), bw_bytes, stream)
            if st != 0:
                raise B.SmileError(st, "smile_layer_backward")

        def timed(fn, nrep):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            c0 = time.perf_counter()
            for _ in range(nrep):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - c0) / nrep

        nrep = max(10, min(steps, 30))
        f_s = timed(fwd_train, nrep)
        b_s = timed(bwd, nrep)
        out["training"] = {"forward_saving_activations_ms": round(f_s * 1e3, 4), "backward_ms": round(b_s * 1e3, 4),
                           "forward_plus_backward_tokens_per_s": round(T / (f_s + b_s), 1),
                           "backward_gemm_tflops": round(8.0 * kept * d * F / b_s / 1e12, 2),
                           "backward_workspace_MB": round(bw_bytes / 1e6, 1)}

    # ---- CPU oracle on the host cores: a bounded sample of the same workload
    cpu = None
    if with_cpu:
        import oracle
        x = wl.gen_tokens(cfg)
        wi, wq = wl.gen_router_weights(cfg)
        bi, bq = wl.gen_routing_biases(cfg)
        thr = oracle.threads()
        budget_flop = 20.0 * 1.5e9 * thr      # about 20 s at the oracle's ~1.5 GFLOP/s per thread
        full_flop = 4.0 * kept * d * F
        if full_flop <= budget_flop:
            w1 = np.stack([wl.gen_expert_weights(cfg, e)[0] for e in range(N)])
            w2 = np.stack([wl.gen_expert_weights(cfg, e)[1] for e in range(N)])
            passes, c0 = 0, time.perf_counter()
            while True:
                oracle.layer_forward(x, wi, wq, w1, w2, cfg.capacity, cfg.act, cfg.dtype, bias_inter=bi, bias_intra=bq)
                passes += 1
                c1 = time.perf_counter()
                if c1 - c0 >= 10.0 or passes >= 64:
                    break
            cpu = {"value": round(passes * T / (c1 - c0), 1), "unit": "tokens/s", "cores": thr, "kind": "oracle",
                   "sample": f"the whole workload {passes} times: all {T} tokens through all steps "
                             f"({c1 - c0:.2f} s in total)"}
        else:
            # routing on all tokens; expert FFN on every stride-th expert (the router is skewed: a prefix of the
            # experts would not be representative), its time scaled by the kept rows covered
            ne = max(1, int(N * budget_flop / full_flop))
            stride = max(1, N // ne)
            picks = list(range(0, N, stride))
            c0 = time.perf_counter()
            li, lq = oracle.gate_logits(x, wi, wq)
            r = oracle.route(li, lq, cfg.capacity, bi, bq)
            xe = oracle.dispatch(x, r.group_idx, r.local_idx, r.slot, n, m, cfg.capacity)
            c1 = time.perf_counter()
            w1 = np.stack([wl.gen_expert_weights(cfg, e)[0] for e in picks])
            w2 = np.stack([wl.gen_expert_weights(cfg, e)[1] for e in picks])
            c2 = time.perf_counter()
            oracle.expert_ffn(xe[picks], r.kept_count[picks], w1, w2, cfg.act, cfg.dtype)
            c3 = time.perf_counter()
            rows = int(r.kept_count[picks].sum())
            kept_o = int(r.kept_count.sum())
            est = (c1 - c0) + (c3 - c2) * kept_o / max(rows, 1)
            cpu = {"value": round(T / est, 1), "unit": "tokens/s", "cores": thr, "kind": "oracle",
                   "sample": f"gate+route+dispatch on all {T} tokens ({c1 - c0:.2f} s), expert FFN on every "
                             f"{stride}th expert ({len(picks)} experts, {rows} of {kept_o} kept rows, "
                             f"{c3 - c2:.2f} s), FFN time extrapolated by rows"}
    layer.close()
    del layer
    torch.cuda.empty_cache()
    return cfg, out, cpu


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="all",
                    help="all (default: headline cfg5, then cfg1..cfg4 under `configs`), or one of cfg1..cfg5, "
                         "t2_48b, cfg4_flat, cfg2_f16 alone")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-backward", action="store_true",
                    help="skip the extra (untimed for `value`) training leg: forward that saves activations + backward")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy (reads 256 MiB, writes 256 MiB) so that a "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE pass of this command has a kernel of known "
                         "traffic to scale the counters by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (all experts resident on one MI355X); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    hip = Hip()
    names = ALL_CONFIGS if args.workload == "all" else [args.workload]
    head_cfg, head, cpu = bench_config(names[0], args.steps, args.warmup, hip, not args.no_backward,
                                       not args.no_cpu_baseline, args.copy_calibration)
    others = {}
    for nm in names[1:]:
        print(f"bench.py: {nm}", file=sys.stderr, flush=True)
        _, res, _ = bench_config(nm, args.steps, args.warmup, hip, False, False)
        others[nm] = res

    out = {
        "metric": "moe_layer_forward_tokens_per_s",
        "value": head["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "ms_per_step_event_median": head["ms_per_step_event_median"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": head_cfg.dtype,
        "data": "synthetic",
        "config": {"workload": head["workload"], "kept_tokens": head["kept_tokens"],
                   "dropped_tokens": head["dropped_tokens"],
                   "max_over_mean_expert_load": head["max_over_mean_expert_load"]},
        "roofline": head["roofline"],
        "expert_gemm_mfma_frac": head["expert_gemm_mfma_frac"],
        "kernels_us": head["kernels_us"],
        "route_kernels_us": head["route_kernels_us"],
        "launches_per_step": head["launches_per_step"],
        "step_minus_kernel_sum_us": head["step_minus_kernel_sum_us"],
        "pre_warm_ms": PRE_WARM_S * 1e3, "pre_warm_steps": head["pre_warm_steps"],
        "hbm": head["hbm"],
        "training": head.get("training"),
        "cpu_baseline": cpu,
        "configs": others,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
