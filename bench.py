#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

A step is one forward + backward pass of the whole path (route, permute, grouped SwiGLU
GEMMs, combine and their backward: every library call of paper_2508_02317_amd.layer) over
one batch of seeded synthetic input that is already resident in HBM.  Prints ONE JSON line.
By default the token rows are gathered inside the grouped products (no expert-ordered copies);
--no-gather times the path with the separate permute / combine-backward launches instead.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline] [--no-gather]

Workloads are the five configurations of paper_2508_02317_amd.inputs.CONFIGS; the default
is the 30B-A3B-class layer on one 8K-token micro-batch ("a3b_8k").
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6     # MI355X dense bf16 MFMA: 256 CU x 2048 MAC/clk x 2 x 2.4 GHz
PEAK_FP32_TFLOPS = 157.3      # fp32 vector
PEAK_HBM_GBS = 8000.0         # HBM3E
PAPER_CONTEXT = ("paper: >2,800 tokens/sec/GPU, 30B MoE, whole model, 128 GPUs (GPU model unstated), "
                 "mixed precision -- context only")

# HBM bytes per launch (read + write) from the `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` runs of this
# command summarised under profiles/, each counter scaled by what it reads for a plain 1 GiB copy
# (fetch x 2.000, write x 1.000).  Keyed by (workload, kernel, rows gathered inside the products); absent = not measured.
MEASURED_TRAFFIC = {
    ("a3b_8k", "combine_fwd", True): 270.1e6 + 33.6e6,
    ("a3b_8k", "ffn_dact", True): 1017.6e6 + 305.6e6,
    ("a3b_8k", "ffn_down", True): 647.5e6 + 268.5e6,
    ("a3b_8k", "ffn_dx", True): 1634.0e6 + 268.5e6,
    ("a3b_8k", "ffn_gate_up", True): 1516.1e6 + 386.6e6,
    ("a3b_8k", "wgrad_down", True): 386.7e6 + 416.1e6,
    ("a3b_8k", "wgrad_gate_up", True): 754.6e6 + 805.7e6,
    ("a3b_8k", "combine_bwd", False): 315.0e6 + 268.7e6,
    ("a3b_8k", "combine_fwd", False): 270.1e6 + 33.6e6,
    ("a3b_8k", "ffn_dact", False): 1084.8e6 + 201.3e6,
    ("a3b_8k", "ffn_down", False): 647.0e6 + 268.5e6,
    ("a3b_8k", "ffn_dx", False): 1627.6e6 + 268.5e6,
    ("a3b_8k", "ffn_gate_up", False): 1551.0e6 + 379.6e6,
    ("a3b_8k", "permute_gather", False): 35.2e6 + 270.1e6,
    ("a3b_8k", "wgrad_down", False): 397.1e6 + 403.5e6,
    ("a3b_8k", "wgrad_gate_up", False): 713.2e6 + 805.6e6,
}


def kernel_work(cfg, P):
    """Algorithmic work per launch of each kernel: ("mfma", flops) or ("hbm", bytes)."""
    T, d, E, k, f = cfg.T, cfg.d, cfg.E, cfg.k, cfg.f
    s = 2 if cfg.dtype == "bf16" else 4
    dff = float(P) * d * f
    mm = "mfma" if cfg.dtype == "bf16" else "alu"
    pre = "ffn_" if cfg.dtype == "bf16" else "f32_"
    work = {
        pre + "gate_up": (mm, 4 * dff), pre + "down": (mm, 2 * dff), pre + "dact": (mm, 2 * dff),
        pre + "dx": (mm, 4 * dff), "wgrad_down": (mm, 2 * dff), "wgrad_gate_up": (mm, 4 * dff),
        "f32_wgrad": (mm, 2 * dff),
        "route_topk": ("hbm", T * E * 4 + P * 8),
        "route_bwd": ("hbm", T * E * 4 + P * 12),
        "permute_gather": ("hbm", (T + P) * d * s + 2 * P * 4),
        "combine_fwd": ("hbm", (P + T) * d * s + P * 8),
        "combine_bwd": ("hbm", (T + 2 * P) * d * s + P * 12),
        # router linear (--router): skinny products, bound by reading / writing the [T, d] side
        "router_logits": ("hbm", T * d * s + E * d * s + T * E * 4),
        "router_cast_dz": ("hbm", T * E * 6),
        "router_dx": ("hbm", 2 * T * d * s + T * E * 2 + E * d * s),
        "wgrad_router": ("hbm", T * d * s + T * E * 2 + E * d * s),
    }
    return work


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="a3b_8k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-save-gu", action="store_true", help="backward recomputes G and U")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time its replays (removes launch overhead; matters "
                         "for the small workloads only)")
    ap.add_argument("--router", action="store_true",
                    help="start from hidden states: the router linear and its backward are part of the step "
                         "(the default step starts from given logits, as the metric's path does)")
    ap.add_argument("--no-gather", action="store_true",
                    help="call moe_permute, moe_grouped_gemm_swiglu_fwd/bwd and moe_unpermute_combine_bwd separately, "
                         "writing the expert-ordered copies xp and dyp (the default step uses the *_gather entry points, "
                         "which read the layer input and the output gradient by token inside the products)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy three times (reference for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (no collectives, no sharding); run with --gpus 1. "
              "`value` is one GPU's throughput.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")       # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel() * 4, "copy_bytes_written": dst.numel() * 4, "launches": 3}))
        return
    from paper_2508_02317_amd import libmoe as L
    from paper_2508_02317_amd.inputs import CONFIGS, make_inputs, select_local_share
    from paper_2508_02317_amd.layer import MoELayer

    cfg = CONFIGS[args.workload]
    torch.cuda.set_device(0)
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    t0 = time.time()
    inp = make_inputs(cfg)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda().to(tdt).contiguous()
    wg, wu, wd = dev(inp["Wg"]), dev(inp["Wu"]), dev(inp["Wd"])
    dy = dev(inp["dY"])
    logits = torch.from_numpy(inp["logits"]).cuda()
    prerouted = cfg.kind == "ep_share"
    if prerouted:
        # route the global problem with the library, cut this GPU's share by pure indexing
        gidx, gw, _, _ = L.moe_route_topk(logits, cfg.k_global, cfg.renorm)
        tok, lidx, lw = select_local_share(gidx.cpu().numpy(), gw.cpu().numpy(), cfg.E, cfg.T)
        assert len(tok) == cfg.T, "global problem too small for the local share"
        Xh = inp["X"][tok]
        x = dev(Xh)
        r_idx, r_w = torch.from_numpy(lidx).cuda(), torch.from_numpy(lw.astype(np.float32)).cuda()
        counts_h = np.bincount(lidx[:, 0], minlength=cfg.E)
        assert counts_h.max() > 5 * (cfg.T_global * cfg.k_global / cfg.E_global), "routing not skewed enough"
    else:
        Xh = inp["X"]
        x = dev(Xh)
    w_router = None
    if args.router:
        assert not prerouted, "--router needs a workload that routes"
        w_router = dev(np.ascontiguousarray(inp["Wr"].T))             # [E, d]
    layer = MoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, tdt, wg, wu, wd, renorm=cfg.renorm, prerouted=prerouted,
                     save_gu=not args.no_save_gu, w_router=w_router, gather=not args.no_gather)
    P = layer.P
    print("[bench] %s: inputs ready in %.1f s" % (cfg.name, time.time() - t0), file=sys.stderr, flush=True)

    def step():
        if prerouted:
            layer.forward(x, topk_idx=r_idx, topk_w=r_w)
            layer.backward(dy)
        else:
            layer.forward(x, logits=logits)
            layer.backward(dy, logits=logits)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    run = step
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        run = graph.replay
        run()
        torch.cuda.synchronize()
    # The per-kernel HIP events (recorded by the library on the launch stream) are taken inside the timed region,
    # on every fifth step: bracketing every launch of every step costs 5 % of the step time at a3b_8k, one step in
    # five costs 1 %.  A graph replay cannot hold events; then they come from a second, eager pass.
    events_in_timed_region = not args.graph
    sample_every = 5
    if events_in_timed_region:
        L.moe_profile_enable(1)
        step()                                     # creates the event pool outside the timed region
        torch.cuda.synchronize()
        L.moe_profile_enable(1)                    # drops those records
        L.moe_profile_enable(0)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(args.steps):
        sampled = events_in_timed_region and i % sample_every == 0
        if sampled:
            L.moe_profile_enable(2)
        run()
        if sampled:
            L.moe_profile_enable(0)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed * 1e3 / args.steps
    tokens_per_s = cfg.T * args.steps / elapsed
    if not events_in_timed_region:
        L.moe_profile_enable(1)
        torch.cuda.synchronize()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
    prof = L.moe_profile_report()
    sclk = L.moe_profile_shader_clock() if cfg.dtype == "bf16" else {}
    L.moe_profile_enable(1)
    L.moe_profile_enable(0)
    sampled_steps = len(range(0, args.steps, sample_every)) if events_in_timed_region else args.steps
    # the same K steps once more without any events, for the record
    torch.cuda.synchronize()
    t_plain = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    ms_per_step_without_events = (time.perf_counter() - t_plain) * 1e3 / args.steps

    work = kernel_work(cfg, P)
    kernels = {}
    for name, (count, total_ms) in prof.items():
        avg_ms = total_ms / count
        entry = {"launches_per_step": count / sampled_steps, "avg_ms": round(avg_ms, 5)}
        if name in work:
            bound, amount = work[name]
            if bound == "hbm":
                entry.update(bound="hbm", achieved=round(amount / (avg_ms * 1e-3) / 1e9, 1), unit="GB/s", peak=PEAK_HBM_GBS)
            else:
                peak = PEAK_BF16_TFLOPS if bound == "mfma" else PEAK_FP32_TFLOPS
                entry.update(bound=bound, achieved=round(amount / (avg_ms * 1e-3) / 1e12, 2), unit="TFLOP/s", peak=peak)
            entry["frac"] = round(entry["achieved"] / entry["peak"], 4)
        if sclk.get(name):
            # shader clock a workgroup in the middle of the launch ran at (nominal 2400 MHz, which `peak` assumes)
            entry["shader_clock_mhz"] = round(sclk[name], 1)
        kernels[name] = entry
    dominant = max((n for n in kernels if "frac" in kernels[n]),
                   key=lambda n: kernels[n]["avg_ms"] * kernels[n]["launches_per_step"])
    dk = kernels[dominant]
    roofline = {"kernel": dominant, "bound": dk["bound"], "achieved": dk["achieved"], "peak": dk["peak"],
                "unit": dk["unit"], "frac": dk["frac"], "avg_ms": dk["avg_ms"],
                "traffic": MEASURED_TRAFFIC.get((cfg.name, dominant, not args.no_gather))}
    if "shader_clock_mhz" in dk:
        roofline["shader_clock_mhz"] = dk["shader_clock_mhz"]
    # everything the two grouped-GEMM entry points launch: the products, the device-side schedules and the
    # reduction of split weight gradients
    gemm_names = [n for n in kernels if kernels[n].get("bound") in ("mfma", "alu") or n.startswith("build_")
                  or n.endswith("_reduce")]
    gemm_ms = sum(kernels[n]["avg_ms"] * kernels[n]["launches_per_step"] for n in gemm_names)
    gemm_tflops = 18.0 * P * cfg.d * cfg.f / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    gemm_peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_FP32_TFLOPS
    # forward / backward separately, and the step against the lower of the two roofs: at about 512 rows per expert
    # the bytes the products cannot avoid (every activation and weight once per product that needs it, the saved
    # and intermediate tensors once each way, the weight gradients once) take as long at 8 TB/s as the flops at peak
    fwd_names = [n for n in gemm_names if n.endswith(("gate_up", "down")) and not n.startswith("wgrad")]
    fwd_ms = sum(kernels[n]["avg_ms"] for n in fwd_names)      # one launch each (a second gate/up launch is the backward's recompute)
    bwd_ms = gemm_ms - fwd_ms - sum(kernels[n]["avg_ms"] * kernels[n]["launches_per_step"] for n in gemm_names if n.startswith("build_"))
    es = 2 if cfg.dtype == "bf16" else 4
    Pd, Pf, Edf = float(P) * cfg.d * es, float(P) * cfg.f * es, float(cfg.E) * cfg.d * cfg.f * es
    fwd_bytes = 2 * Pd + 2 * Pf + 3 * Edf + (0 if args.no_save_gu else 2 * Pf)      # x, act out + in, yp; weights; G, U
    bwd_bytes = 3 * Pd + 3 * Pf + 4 * Pf + 6 * Edf      # dy, x, dxp; act, G, U; [dG|dU] out + in; weights in, gradients out
    hbm_floor_ms = (fwd_bytes + bwd_bytes) / (PEAK_HBM_GBS * 1e9) * 1e3
    mfma_floor_ms = 18.0 * P * cfg.d * cfg.f / (gemm_peak * 1e12) * 1e3

    working_set = 6 * Edf + 4 * float(cfg.T) * cfg.d * es + 3 * Pd + 6 * Pf
    out = {
        "metric": "MoE layer fwd+bwd tokens/sec on 1 MI355X; grouped-GEMM % of bf16 MFMA peak",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_per_step_without_events": round(ms_per_step_without_events, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "T": cfg.T, "d": cfg.d, "E": cfg.E, "k": cfg.k, "f": cfg.f, "P": P,
                   "renorm": cfg.renorm, "save_gu": not args.no_save_gu, "router_linear_in_step": bool(args.router), "hip_graph": bool(args.graph),
                   "gather_in_gemm": not args.no_gather,
                   "kernel_events": ("every %dth timed step" % sample_every) if events_in_timed_region else "second pass",
                   "unit_note": "routed rows/s" if prerouted else "tokens/s",
                   # weights and their gradients, the token-major and the expert-ordered activations: under 256 MB the
                   # step runs out of the last-level cache and its mover GB/s are not HBM rates
                   "working_set_mb": round(working_set / 1e6, 1), "cache_resident": bool(working_set < 256e6)},
        "roofline": roofline,
        "grouped_gemm": {"tflops": round(gemm_tflops, 2), "frac_of_peak": round(gemm_tflops / gemm_peak, 4),
                         "peak": gemm_peak, "ms_per_step": round(gemm_ms, 4),
                         "fwd_tflops": round(6.0 * P * cfg.d * cfg.f / (fwd_ms * 1e-3) / 1e12, 2) if fwd_ms > 0 else None,
                         "bwd_tflops": round(12.0 * P * cfg.d * cfg.f / (bwd_ms * 1e-3) / 1e12, 2) if bwd_ms > 0 else None,
                         "mfma_floor_ms": round(mfma_floor_ms, 4), "hbm_floor_ms": round(hbm_floor_ms, 4),
                         "frac_of_lower_roof": round(max(mfma_floor_ms, hbm_floor_ms) / gemm_ms, 4) if gemm_ms > 0 else None},
        "kernels": kernels,
        "context": PAPER_CONTEXT,
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, inp, Xh, layer, prerouted,
                                           (lidx, lw) if prerouted else None)
    print(json.dumps(out), flush=True)


def cpu_baseline(cfg, inp, Xh, layer, prerouted, routing):
    """The fp64 oracle, as it stands, timed on the host cores on a bounded sample: the
    first Ts tokens of the same workload (tokens are independent in the forward, so its Y
    and dX rows are also a parity check of the GPU result)."""
    import numpy as np
    from oracle import moe_oracle as O
    flops_per_token = 18.0 * cfg.d * cfg.f * cfg.k
    Ts = int(min(cfg.T, max(64, 1.0e13 // flops_per_token)))      # at most 10 TFLOP of fp64 work (about 20 s on 16 host cores)
    X, dY = Xh[:Ts], inp["dY"][:Ts]
    t0 = time.perf_counter()
    if prerouted:
        fwd = O.moe_layer_fwd(X, None, inp["Wg"], inp["Wu"], inp["Wd"], 1,
                              routing=(routing[0][:Ts], routing[1][:Ts].astype(np.float32)))
        bwd = O.moe_layer_bwd(fwd, dY, None, inp["Wg"], inp["Wu"], inp["Wd"])
    else:
        z = inp["logits"][:Ts]
        fwd = O.moe_layer_fwd(X, z, inp["Wg"], inp["Wu"], inp["Wd"], cfg.k, cfg.renorm)
        bwd = O.moe_layer_bwd(fwd, dY, z, inp["Wg"], inp["Wu"], inp["Wd"], cfg.renorm)
    dt = time.perf_counter() - t0
    y = layer.y[:Ts].float().cpu().numpy().astype(np.float64)
    dx = layer.dx[:Ts].float().cpu().numpy().astype(np.float64)
    err_y = float(np.max(np.abs(y - fwd["Y"])) / np.max(np.abs(fwd["Y"])))
    err_dx = float(np.max(np.abs(dx - bwd["dX"])) / np.max(np.abs(bwd["dX"])))
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    return {"value": round(Ts / dt, 1), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": "first %d of %d tokens, full fwd+bwd in numpy fp64 (%.1f s)" % (Ts, cfg.T, dt),
            "host_cores_available": len(os.sched_getaffinity(0)),
            "parity_on_sample": {"Y": err_y, "dX": err_dx}}


if __name__ == "__main__":
    main()
