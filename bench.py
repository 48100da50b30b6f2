#!/usr/bin/env python3
"""Benchmark of the SMILE bi-level MoE layer forward on one MI355X.

One "step" is one pass of the whole hot path over one batch of seeded synthetic tokens: gate
logits -> bi-level routing with capacity -> dispatch -> expert FFN (up, down) -> combine -> LB loss,
all through the C-ABI library, inputs and weights resident in HBM.  The workload is the
Switch-base-shaped bf16 configuration (T=8192, d=768, F=3072, 2 groups x 8 experts, cf 1.0).

Prints ONE JSON line: tokens/s of the whole layer (timed region: K calls of smile_layer_forward),
the roofline of the dominant kernel (the up-projection + GELU grouped GEMM, timed inside the timed
region with a HIP event pair that the library attaches to that kernel's launch on its stream),
per-step times from a second, instrumented pass over the six separate entry points, a third pass
that times a training step (forward that saves activations, then the backward pass), and the CPU
oracle timed on the host cores.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 / fp16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E

# HBM bytes per launch of the dominant kernel (up-projection GEMM) from the two rocprofv3 --pmc passes
# summarised in profiles/bench_cfg2_hbm_traffic_pmc.txt: FETCH_SIZE 43040.8 KiB x 1.99981 + WRITE_SIZE
# 48024.0 KiB x 1.00000 (scale factors = what the same counters read for a plain 256 MiB device copy).
# Measured for the headline workload only.
MEASURED_TRAFFIC_BYTES = {"cfg2": 137.32e6}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2", help="cfg1..cfg5 (cfg2 is the headline workload), t2_48b, cfg4_flat or cfg2_f16")
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

    import numpy as np
    import torch
    from paper_2212_05191_amd import binding as B
    from paper_2212_05191_amd import workloads as wl
    from paper_2212_05191_amd.runner import GpuLayer

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    lib = B.load()
    cfg = wl.get_config(args.workload)
    layer = GpuLayer(cfg, workers=16)
    b, h = layer.buf, layer.ctx.handle
    stream = torch.cuda.current_stream().cuda_stream
    p = B._ptr

    # pre-marshalled step-by-step calls for the instrumented pass: (name, function, args)
    calls = [
        ("gate_logits", lib.smile_gate_logits,
         (h, p(layer.x), p(layer.w_inter), p(layer.w_intra), p(b.logits_inter), p(b.logits_intra), stream)),
        ("route_bilevel", lib.smile_route_bilevel,
         (h, p(b.logits_inter), p(b.logits_intra), p(layer.bias_inter), p(layer.bias_intra), p(b.group_idx),
          p(b.local_idx), p(b.pos_in_group), p(b.slot), p(b.gate), p(b.p_top), p(b.q_top), p(b.group_count),
          p(b.local_count), p(b.expert_count), p(b.kept_count), p(b.p_sum), p(b.q_sum), stream)),
        ("dispatch", lib.smile_dispatch,
         (h, p(layer.x), p(b.group_idx), p(b.local_idx), p(b.slot), p(b.xe), stream)),
        ("expert_ffn_up", lib.smile_expert_ffn_up,
         (h, p(b.xe), p(b.kept_count), p(layer.w1), None, stream)),
        ("expert_ffn_down", lib.smile_expert_ffn_down,
         (h, p(b.kept_count), p(layer.w2), None, p(b.ye), stream)),
        ("combine", lib.smile_combine,
         (h, p(b.ye), p(b.group_idx), p(b.local_idx), p(b.slot), p(b.gate), p(b.y), stream)),
        ("aux_loss", lib.smile_aux_loss,
         (h, p(b.group_count), p(b.local_count), p(b.p_sum), p(b.q_sum), p(b.loss3), stream)),
    ]
    dominant = 3   # expert_ffn_up

    # raw HIP events (timing enabled) for the dominant kernel: the library passes them to the
    # launch itself, so they carry the kernel's own begin / end timestamps on its stream
    hip = ctypes.CDLL("libamdhip64.so")

    def new_event():
        e = ctypes.c_void_p()
        assert hip.hipEventCreate(ctypes.byref(e)) == 0
        return e

    def elapsed_ms(a, z):
        ms = ctypes.c_float()
        assert hip.hipEventElapsedTime(ctypes.byref(ms), a, z) == 0
        return float(ms.value)

    io = layer.io_fused     # no expert buffers: dispatch / combine fused into the expert GEMMs

    def step(ev=None):
        """One forward pass through the single chained entry point (all steps, fewest launches)."""
        io.prof_up_start, io.prof_up_stop = (ev[0], ev[1]) if ev is not None else (None, None)
        st = lib.smile_layer_forward(h, ctypes.byref(io), stream)
        if st != 0:
            raise B.SmileError(st, "smile_layer_forward")

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps, one event pair per step around the dominant kernel
    evs = [(new_event(), new_event()) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(evs[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    sec_per_step = (t1 - t0) / args.steps
    dom_ms = float(np.mean([elapsed_ms(a, z) for a, z in evs]))
    for a, z in evs:
        hip.hipEventDestroy(a)
        hip.hipEventDestroy(z)

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    kept = int(b.kept_count.sum().item())
    dropped = cfg.T - kept
    ecnt = b.expert_count.cpu().numpy()
    s = 4 if cfg.dtype == "f32" else 2
    d, F, T, N = cfg.d_model, cfg.d_ff, cfg.T, cfg.N
    up_flops = 2.0 * kept * d * F
    achieved_tflops = up_flops / (dom_ms * 1e-3) / 1e12

    # ---- second, instrumented pass (not part of `value`): events around every call
    nrep = max(10, min(args.steps, 50))
    marks = [[torch.cuda.Event(enable_timing=True) for _ in range(len(calls) + 1)] for _ in range(nrep)]
    torch.cuda.synchronize()
    for r in range(nrep):
        marks[r][0].record()
        for i, (name, fn, a) in enumerate(calls):
            fn(*a)
            marks[r][i + 1].record()
    torch.cuda.synchronize()
    per_call_us = {name: 1e3 * float(np.median([marks[r][i].elapsed_time(marks[r][i + 1]) for r in range(nrep)]))
                   for i, (name, _, _) in enumerate(calls)}
    alg_bytes = {
        "gate_logits": T * d * s + (cfg.n_groups + cfg.m_local) * d * s + 4 * T * (cfg.n_groups + cfg.m_local),
        "dispatch": 2 * kept * d * s + 12 * T,
        "combine": kept * d * s + T * d * s + 16 * T,
        "expert_ffn_up": N * d * F * s + kept * d * s + kept * F * s,
        "expert_ffn_down": N * d * F * s + kept * F * s + kept * d * s,
    }
    hbm = {k: {"us": round(per_call_us[k], 2), "alg_MB": round(v / 1e6, 2),
               "GBps": round(v / (per_call_us[k] * 1e-6) / 1e9, 1),
               "frac_of_8TBps": round(v / (per_call_us[k] * 1e-6) / 1e9 / PEAK_HBM_GBS, 4)}
           for k, v in alg_bytes.items()}
    down_tflops = up_flops / (per_call_us["expert_ffn_down"] * 1e-6) / 1e12

    # ---- third pass (not part of `value`): training step = forward with expert buffers and saved
    # activations, then the backward pass, each through its single chained entry point
    train = None
    if not args.no_backward:
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

        def timed(fn, reps):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            c0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - c0) / reps

        reps = max(10, min(args.steps, 30))
        f_s = timed(fwd_train, reps)
        b_s = timed(bwd, reps)
        bwd_flops = 8.0 * kept * d * F      # the four gradient GEMMs (dh, dxe, dW1, dW2)
        train = {"forward_saving_activations_ms": round(f_s * 1e3, 4), "backward_ms": round(b_s * 1e3, 4),
                 "forward_plus_backward_tokens_per_s": round(T / (f_s + b_s), 1),
                 "backward_gemm_tflops": round(bwd_flops / b_s / 1e12, 2),
                 "backward_workspace_MB": round(bw_bytes / 1e6, 1)}

    # ---- CPU oracle on the host cores (same workload, one pass)
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        x = wl.gen_tokens(cfg)
        wi, wq = wl.gen_router_weights(cfg)
        bi, bq = wl.gen_routing_biases(cfg)
        # bound the CPU work to roughly 10-30 s: the oracle does about 1.5 GFLOP/s per thread
        thr = oracle.threads()
        budget_flop = 20.0 * 1.5e9 * thr
        full_flop = 4.0 * kept * d * F
        if full_flop <= budget_flop:
            w1 = np.stack([wl.gen_expert_weights(cfg, e)[0] for e in range(N)])
            w2 = np.stack([wl.gen_expert_weights(cfg, e)[1] for e in range(N)])
            # whole passes of the workload until about 10 s of CPU work have been timed
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
            # routing on all tokens, expert FFN on the first experts only; scale the FFN time up
            ne = max(1, int(N * budget_flop / full_flop))
            c0 = time.perf_counter()
            li, lq = oracle.gate_logits(x, wi, wq)
            r = oracle.route(li, lq, cfg.capacity, bi, bq)
            xe = oracle.dispatch(x, r.group_idx, r.local_idx, r.slot, cfg.n_groups, cfg.m_local, cfg.capacity)
            c1 = time.perf_counter()
            w1 = np.stack([wl.gen_expert_weights(cfg, e)[0] for e in range(ne)])
            w2 = np.stack([wl.gen_expert_weights(cfg, e)[1] for e in range(ne)])
            c2 = time.perf_counter()
            ye = oracle.expert_ffn(xe[:ne], r.kept_count[:ne], w1, w2, cfg.act, cfg.dtype)
            c3 = time.perf_counter()
            rows = int(r.kept_count[:ne].sum())
            est = (c1 - c0) + (c3 - c2) * kept / max(rows, 1)
            cpu = {"value": round(T / est, 1), "unit": "tokens/s", "cores": thr, "kind": "oracle",
                   "sample": f"gate+route+dispatch on all {T} tokens, expert FFN on experts 0..{ne - 1} "
                             f"({rows} of {kept} kept rows), FFN time extrapolated by rows"}

    out = {
        "metric": "moe_layer_forward_tokens_per_s",
        "value": round(T / sec_per_step, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={T} d_model={d} d_ff={F} experts={cfg.n_groups}x{cfg.m_local} "
                               f"capacity={cfg.capacity} (cf {cfg.capacity_factor}) {cfg.dtype} {cfg.act}",
                   "kept_tokens": kept, "dropped_tokens": dropped,
                   "max_over_mean_expert_load": round(float(ecnt.max() / max(ecnt.mean(), 1e-9)), 3)},
        "roofline": {"kernel": "grouped_gemm_nt_kernel (expert FFN up-projection + GELU)",
                     "bound": "mfma", "achieved": round(achieved_tflops, 2), "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved_tflops / PEAK_BF16_TFLOPS, 4),
                     "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name), "avg_launch_us": round(dom_ms * 1e3, 2),
                     "alg_flops_per_launch": up_flops},
        "expert_ffn_down_tflops": round(down_tflops, 2),
        "expert_gemm_mfma_frac": round((2 * up_flops) / ((per_call_us["expert_ffn_up"] + per_call_us["expert_ffn_down"])
                                                         * 1e-6) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "steps_us": {k: round(v, 2) for k, v in per_call_us.items()},
        "hbm": hbm,
        "training": train,
        "cpu_baseline": cpu,
    }
    layer.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
