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

Timing: `ms_per_step` is the wall clock over the K timed steps between two device
synchronisations; `ms_per_step_median` is the median of the K per-step intervals between HIP
events recorded on the launch stream at the step boundaries.  Per-kernel and per-entry-point
durations come from HIP events that this script records, through the library's launch hook, on
the stream each kernel is launched on, in every fifth step of the same timed region.
"""
import argparse
import ctypes
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6     # MI355X dense bf16 MFMA: 256 CU x 2048 MAC/clk x 2 x 2.4 GHz
PEAK_FP32_TFLOPS = 157.3      # fp32 vector
PEAK_FP8_TFLOPS = 5033.2      # dense fp8 MFMA (twice the bf16 rate)
PEAK_HBM_GBS = 8000.0         # HBM3E
PAPER_CONTEXT = ("paper: >2,800 tokens/sec/GPU, 30B MoE, whole model, 128 GPUs (GPU model unstated), "
                 "mixed precision -- context only")
SAMPLE_EVERY = 5              # steps between two steps whose launches are bracketed by events


def kernel_work(cfg, P, gather, save_gu, late_weight=False):
    """Per kernel: (bound, algorithmic amount per launch, compulsory HBM bytes per launch or None).

    Flops count routed work only.  The compulsory bytes of a product are its operands read once and its
    results written once (what it would move with perfect reuse inside the launch); their sum over the
    products is the HBM floor of the grouped GEMMs."""
    T, d, E, k, f = cfg.T, cfg.d, cfg.E, cfg.k, cfg.f
    s = 2 if cfg.dtype == "bf16" else 4
    dff = float(P) * d * f
    Pd, Pf, Edf = float(P) * d * s, float(P) * f * s, float(E) * d * f * s
    Td = float(T) * d * s
    xin = Td if gather else Pd          # the gathered products read the token-major matrix
    mm = "mfma" if cfg.dtype == "bf16" else "alu"
    pre = "ffn_" if cfg.dtype == "bf16" else "f32_"
    gu_out = (3 if save_gu else 1) * Pf
    work = {
        pre + "gate_up": (mm, 4 * dff, xin + 2 * Edf + gu_out),
        pre + "down": (mm, 2 * dff, Pf + Edf + Pd),
        pre + "dact": (mm, 2 * dff, xin + Edf + 2 * Pf + 2 * Pf + (Pf if late_weight else 0)),   # + w * act out if the forward did not write it
        pre + "dx": (mm, 4 * dff, 2 * Pf + 2 * Edf + Pd),
        "wgrad_down": (mm, 2 * dff, xin + Pf + Edf),
        "wgrad_gate_up": (mm, 4 * dff, 2 * Pf + xin + 2 * Edf),
        "f32_wgrad": (mm, 2 * dff, None),
        "route_topk": ("hbm", T * E * 4 + P * 8, None),
        "route_bwd": ("hbm", T * E * 4 + P * 12, None),
        "permute_gather": ("hbm", (T + P) * d * s + 2 * P * 4, None),
        "combine_fwd": ("hbm", (P + T) * d * s + P * 8, None),
        "combine_bwd": ("hbm", (T + 2 * P) * d * s + P * 12, None),
        # router linear (--router): skinny products, bound by reading / writing the [T, d] side
        "router_logits": ("hbm", T * d * s + E * d * s + T * E * 4, None),
        "router_cast_dz": ("hbm", T * E * 6, None),
        "router_dx": ("hbm", 2 * T * d * s + T * E * 2 + E * d * s, None),
        "wgrad_router": ("hbm", T * d * s + T * E * 2 + E * d * s, None),
    }
    return work


def measured_traffic(workload, gather):
    """HBM bytes per launch (read + write) of each kernel from the `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE`
    summary of this workload under profiles/ (lines `traffic <kernel> <read MB> <write MB>`), with the file they
    come from; ({}, None) when the workload has no summary."""
    rel = os.path.join("profiles", workload + ("" if gather else "_no_gather") + ".md")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return {}, None
    out = {}
    for m in re.finditer(r"^traffic\s+(\S+)\s+([0-9.]+)\s+([0-9.]+)\s*$", open(path).read(), flags=re.M):
        out[m.group(1)] = (float(m.group(2)) + float(m.group(3))) * 1e6
    return out, rel


class HipEvents:
    """hipEvent_t through ctypes, from the HIP runtime this process has already loaded."""

    def __init__(self):
        path = None
        for line in open("/proc/self/maps"):
            if "libamdhip64" in line:
                path = line.split()[-1]
                break
        if path is None:
            raise RuntimeError("no HIP runtime loaded in this process")
        self.hip = ctypes.CDLL(path)
        vp = ctypes.c_void_p
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(vp)]
        self.hip.hipEventRecord.argtypes = [vp, vp]
        self.hip.hipEventSynchronize.argtypes = [vp]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), vp, vp]
        self.pool = []

    def _ok(self, rc, what):
        if rc != 0:
            raise RuntimeError("%s failed with HIP status %d" % (what, rc))

    def reserve(self, n):
        while len(self.pool) < n:
            ev = ctypes.c_void_p()
            self._ok(self.hip.hipEventCreate(ctypes.byref(ev)), "hipEventCreate")
            self.pool.append(ev)

    def record(self, stream):
        if not self.pool:
            self.reserve(64)
        ev = self.pool.pop()
        self._ok(self.hip.hipEventRecord(ev, ctypes.c_void_p(stream)), "hipEventRecord")
        return ev

    def elapsed_ms(self, a, b):
        self._ok(self.hip.hipEventSynchronize(b), "hipEventSynchronize")
        ms = ctypes.c_float()
        self._ok(self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b), "hipEventElapsedTime")
        return float(ms.value)

    def release(self, evs):
        self.pool.extend(evs)


class LaunchTimer:
    """Brackets every kernel launch of the library with events on the launch stream; an entry point's interval
    runs from the start event of its first kernel to the stop event of its last."""

    def __init__(self, L, events):
        self.L, self.ev = L, events
        self.kernels, self.exports = [], []      # (name, start event, stop event)
        self._open_k = self._open_e = None
        self.hook = L.LAUNCH_HOOK(self._on_launch)

    def _on_launch(self, name, phase, stream, user):
        if phase == 0:
            self._open_k = (name, self.ev.record(stream))
        elif phase == 1:
            self.kernels.append((self._open_k[0].decode(), self._open_k[1], self.ev.record(stream)))
        elif phase == 2:
            self._open_e = len(self.kernels)
        elif len(self.kernels) > self._open_e:
            self.exports.append((name.decode(), self.kernels[self._open_e][1], self.kernels[-1][2]))

    def __enter__(self):
        self.L.moe_set_launch_hook(self.hook)
        return self

    def __exit__(self, *exc):
        self.L.moe_set_launch_hook(None)
        return False

    def report(self):
        """-> ({kernel: (launches, total ms)}, {entry point: (calls, total ms)}) and forgets the records."""
        out = []
        for recs in (self.kernels, self.exports):
            agg = {}
            for name, a, b in recs:
                n, ms = agg.get(name, (0, 0.0))
                agg[name] = (n + 1, ms + self.ev.elapsed_ms(a, b))
            out.append(agg)
        for _, a, b in self.kernels:
            self.ev.release([a, b])
        self.kernels.clear()
        self.exports.clear()
        return out


def mx8_forward_leg(cfg, layer, x, wg, wu, wd, L, events, steps, warmup):
    """The expert forward with 8-bit block-scaled operands (MXFP8), as a separate leg: quantise the layer input, then
    the two products (rows read by token; the activation is quantised inside the first product).  The weights are
    quantised once outside the timed region -- they change once per optimiser step, not per micro-batch -- and that
    cost is reported beside it.  The routing of the bf16 step just run is reused."""
    import torch
    P, d, f, E = layer.P, cfg.d, cfg.f, cfg.E
    stream = torch.cuda.current_stream().cuda_stream
    timer = LaunchTimer(L, events)
    torch.cuda.synchronize()
    with timer:
        wq = [L.moe_mx8_quantise(w) for w in (wg, wu, wd)]
    torch.cuda.synchronize()
    wprof, _ = timer.report()
    xq = L.moe_mx8_quantise(x)
    out = L.moe_grouped_gemm_swiglu_fwd_mx8(xq[0], xq[1], wq[0][0], wq[0][1], wq[1][0], wq[1][1], wq[2][0], wq[2][1], layer.offsets,
                                            pair_of_row=layer.pair_of_row, k=cfg.k)
    ws = torch.empty(L.lib.moe_grouped_gemm_swiglu_fwd_mx8_workspace_bytes(P, d, f, E), dtype=torch.uint8, device=x.device)

    def fwd():
        L.moe_mx8_quantise(x, out=xq)
        L.moe_grouped_gemm_swiglu_fwd_mx8(xq[0], xq[1], wq[0][0], wq[0][1], wq[1][0], wq[1][1], wq[2][0], wq[2][1], layer.offsets,
                                          pair_of_row=layer.pair_of_row, k=cfg.k, out=out, ws=ws)
    for _ in range(warmup):
        fwd()
    torch.cuda.synchronize()
    a = events.record(stream)
    for i in range(steps):
        if i % SAMPLE_EVERY == 0:
            with timer:
                fwd()
        else:
            fwd()
    b = events.record(stream)
    ms = events.elapsed_ms(a, b) / steps
    events.release([a, b])
    prof, _ = timer.report()
    dff = float(P) * d * f
    flops = {"ffn_gate_up_mx8": 4 * dff, "ffn_down_mx8": 2 * dff}
    kernels = {}
    for name, (count, total) in prof.items():
        avg = total / count
        kernels[name] = {"avg_ms": round(avg, 5)}
        if name in flops:
            tf = flops[name] / (avg * 1e-3) / 1e12
            kernels[name].update(bound="mfma", achieved=round(tf, 2), unit="TFLOP/s", peak=PEAK_FP8_TFLOPS, frac=round(tf / PEAK_FP8_TFLOPS, 4))
        elif name == "mx8_quantise":
            gbs = 3.0 * cfg.T * d / (avg * 1e-3) / 1e9          # 2 bytes read, 1 written per element
            kernels[name].update(bound="hbm", achieved=round(gbs, 1), unit="GB/s", peak=PEAK_HBM_GBS, frac=round(gbs / PEAK_HBM_GBS, 4))
    gemm_ms = sum(kernels[n]["avg_ms"] for n in flops if n in kernels)
    return {"what": "expert forward (x quantise + gate/up + down) with MXFP8 operands, fp32 accumulation; never part of `value`",
            "ms_per_forward": round(ms, 4), "kernels": kernels,
            "grouped_gemm": {"ms": round(gemm_ms, 4), "tflops": round(6 * dff / (gemm_ms * 1e-3) / 1e12, 2),
                             "frac_of_peak": round(6 * dff / (gemm_ms * 1e-3) / 1e12 / PEAK_FP8_TFLOPS, 4), "peak": PEAK_FP8_TFLOPS},
            "weight_quantise_ms_outside_timed_region": round(sum(t for _, t in wprof.values()), 4)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=None,
                    help="one of the five configurations; default a3b_8k (the configuration the metric is quoted on), followed by a "
                         "short run of each of the other four whose summaries go into `other_workloads` of the same line")
    ap.add_argument("--no-others", action="store_true", help="default run only: skip the short runs of the other four configurations")
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
    ap.add_argument("--weight-in-combine", action="store_true",
                    help="gathered step only: leave the combine weight to moe_unpermute_combine_fwd (the backward then forms and "
                         "stores w * act itself); the default applies it inside the forward products")
    ap.add_argument("--no-mx8", action="store_true", help="skip the separate 8-bit forward leg (key `mx8_forward` of the line)")
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
    headline = args.workload or "a3b_8k"
    out = measure(args, headline)
    if args.workload is None and not args.no_others:
        # The other configurations, briefly (no oracle leg, no 8-bit leg, fewer steps): summaries only.  The full lines
        # come from `bench.py --workload <name>` and live in profiles/.
        import copy
        import gc
        import torch as _torch
        brief = copy.copy(args)
        brief.no_cpu_baseline, brief.no_mx8 = True, True
        brief.steps, brief.warmup = min(args.steps, 20), min(args.warmup, 5)
        others = {}
        for name in ("a3b_long", "a3b_ep_skew", "small", "tiny"):
            gc.collect()
            _torch.cuda.empty_cache()
            o = measure(brief, name)
            others[name] = {"ms_per_step_median": o["ms_per_step_median"], "value": o["value"], "unit": o["config"]["unit_note"],
                            "steps": o["steps"], "dtype": o["dtype"], "cache_resident": o["config"]["cache_resident"],
                            "grouped_gemm_tflops": o["grouped_gemm"]["tflops"], "grouped_gemm_frac_of_peak": o["grouped_gemm"]["frac_of_peak"],
                            "roofline": o["roofline"], "small_launches_ms_per_step": o["small_launches_ms_per_step"]}
        out["other_workloads"] = others
    print(json.dumps(out), flush=True)


def measure(args, workload):
    """One workload: inputs, warm-up, the timed steps, per-kernel events -> the dict of the bench line."""
    import numpy as np
    import torch
    from paper_2508_02317_amd import libmoe as L
    from paper_2508_02317_amd.inputs import CONFIGS, make_inputs, select_local_share
    from paper_2508_02317_amd.layer import MoELayer

    cfg = CONFIGS[workload]
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
    gather, save_gu = not args.no_gather, not args.no_save_gu
    layer = MoELayer(cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, tdt, wg, wu, wd, renorm=cfg.renorm, prerouted=prerouted,
                     save_gu=save_gu, w_router=w_router, gather=gather,
                     weight_in_forward=(gather and not args.weight_in_combine))
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

    events = HipEvents()
    timer = LaunchTimer(L, events)
    # A graph replay cannot call the hook; then the per-kernel events come from a second, eager pass.
    events_in_timed_region = not args.graph
    with timer:                                    # one sampled step outside the timed region: sizes the event pool
        step()
    torch.cuda.synchronize()
    per_step = 2 * len(timer.kernels)
    timer.report()
    n_sampled = len(range(0, args.steps, SAMPLE_EVERY)) if events_in_timed_region else args.steps
    events.reserve(per_step * n_sampled + args.steps + 8)
    stream = torch.cuda.current_stream().cuda_stream

    torch.cuda.synchronize()
    marks = [events.record(stream)]
    t_start = time.perf_counter()
    for i in range(args.steps):
        if events_in_timed_region and i % SAMPLE_EVERY == 0:
            with timer:
                run()
        else:
            run()
        marks.append(events.record(stream))
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed * 1e3 / args.steps
    tokens_per_s = cfg.T * args.steps / elapsed
    step_ms = [events.elapsed_ms(marks[i], marks[i + 1]) for i in range(args.steps)]
    events.release(marks)
    if not events_in_timed_region:
        with timer:
            for _ in range(args.steps):
                step()
        torch.cuda.synchronize()
    prof, exports_prof = timer.report()
    # the same K steps once more with no hook at all, for the record
    torch.cuda.synchronize()
    t_plain = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    ms_per_step_without_events = (time.perf_counter() - t_plain) * 1e3 / args.steps

    work = kernel_work(cfg, P, gather, save_gu, late_weight=gather and not layer.weight_in_forward)
    traffic, traffic_source = measured_traffic(cfg.name, gather) if (save_gu and not args.router) else ({}, None)
    kernels = {}
    for name, (count, total_ms) in prof.items():
        avg_ms = total_ms / count
        entry = {"launches_per_step": count / n_sampled, "avg_ms": round(avg_ms, 5)}
        if name in work:
            bound, amount, floor_bytes = work[name]
            if bound == "hbm":
                entry.update(bound="hbm", achieved=round(amount / (avg_ms * 1e-3) / 1e9, 1), unit="GB/s", peak=PEAK_HBM_GBS)
            else:
                peak = PEAK_BF16_TFLOPS if bound == "mfma" else PEAK_FP32_TFLOPS
                entry.update(bound=bound, achieved=round(amount / (avg_ms * 1e-3) / 1e12, 2), unit="TFLOP/s", peak=peak)
                if floor_bytes:
                    entry["compulsory_mb"] = round(floor_bytes / 1e6, 1)
            entry["frac"] = round(entry["achieved"] / entry["peak"], 4)
        if name in traffic:
            entry["traffic"] = traffic[name]
        kernels[name] = entry
    dominant = max((n for n in kernels if "frac" in kernels[n]),
                   key=lambda n: kernels[n]["avg_ms"] * kernels[n]["launches_per_step"])
    dk = kernels[dominant]
    roofline = {"kernel": dominant, "bound": dk["bound"], "achieved": dk["achieved"], "peak": dk["peak"],
                "unit": dk["unit"], "frac": dk["frac"], "avg_ms": dk["avg_ms"],
                "traffic": traffic.get(dominant), "traffic_source": traffic_source if dominant in traffic else None}
    # everything the two grouped-GEMM entry points launch: the products, the device-side schedules and the
    # reduction of split weight gradients
    gemm_names = [n for n in kernels if kernels[n].get("bound") in ("mfma", "alu") or n.startswith("build_")
                  or n.endswith("_reduce") or n == "finish_dw"]
    gemm_ms = sum(kernels[n]["avg_ms"] * kernels[n]["launches_per_step"] for n in gemm_names)
    gemm_tflops = 18.0 * P * cfg.d * cfg.f / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    gemm_peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_FP32_TFLOPS
    # forward / backward separately, and the step against the lower of the two roofs: at about 512 rows per expert the
    # bytes the products cannot avoid take as long at 8 TB/s as the flops at peak
    fwd_names = [n for n in gemm_names if n.endswith(("gate_up", "down")) and not n.startswith("wgrad")]
    fwd_ms = sum(kernels[n]["avg_ms"] for n in fwd_names)      # one launch each (a second gate/up launch is the backward's recompute)
    bwd_ms = gemm_ms - fwd_ms - sum(kernels[n]["avg_ms"] * kernels[n]["launches_per_step"] for n in gemm_names if n.startswith("build_"))
    floor_bytes = sum(work[n][2] * kernels[n]["launches_per_step"] for n in gemm_names if n in work and work[n][2])
    hbm_floor_ms = floor_bytes / (PEAK_HBM_GBS * 1e9) * 1e3
    mfma_floor_ms = 18.0 * P * cfg.d * cfg.f / (gemm_peak * 1e12) * 1e3
    # launches that are neither products nor movers: routing book-keeping, schedules, small reductions
    small = [n for n in kernels if "frac" not in kernels[n] or n in ("route_topk", "route_bwd")]
    small_ms = sum(kernels[n]["avg_ms"] * kernels[n]["launches_per_step"] for n in small)

    es = 2 if cfg.dtype == "bf16" else 4
    Pd, Pf, Edf = float(P) * cfg.d * es, float(P) * cfg.f * es, float(cfg.E) * cfg.d * cfg.f * es
    working_set = 6 * Edf + 4 * float(cfg.T) * cfg.d * es + 3 * Pd + 6 * Pf
    out = {
        "metric": "MoE layer fwd+bwd tokens/sec on 1 MI355X; grouped-GEMM % of bf16 MFMA peak",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_per_step_median": round(statistics.median(step_ms), 4),
        "ms_per_step_min": round(min(step_ms), 4), "ms_per_step_max": round(max(step_ms), 4),
        "ms_per_step_without_events": round(ms_per_step_without_events, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "T": cfg.T, "d": cfg.d, "E": cfg.E, "k": cfg.k, "f": cfg.f, "P": P,
                   "renorm": cfg.renorm, "save_gu": save_gu, "router_linear_in_step": bool(args.router), "hip_graph": bool(args.graph),
                   "gather_in_gemm": gather, "combine_weight_in_forward_products": bool(layer.weight_in_forward),
                   "kernel_events": ("every %dth timed step" % SAMPLE_EVERY) if events_in_timed_region else "second pass",
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
        "small_launches_ms_per_step": round(small_ms, 4),
        "kernels": kernels,
        "entry_points": {n: {"calls_per_step": c / n_sampled, "avg_ms": round(ms / c, 5)} for n, (c, ms) in exports_prof.items()},
        "traffic_source": traffic_source,
        "context": PAPER_CONTEXT,
    }

    if not args.no_mx8 and cfg.dtype == "bf16" and cfg.d % 128 == 0 and cfg.f % 128 == 0:
        bf16_fwd = sum(kernels[n]["avg_ms"] for n in ("ffn_gate_up", "ffn_down") if n in kernels)
        out["mx8_forward"] = mx8_forward_leg(cfg, layer, x, wg, wu, wd, L, events, args.steps, args.warmup)
        out["mx8_forward"]["bf16_products_ms_for_comparison"] = round(bf16_fwd, 4)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, inp, Xh, layer, prerouted,
                                           (lidx, lw) if prerouted else None)
    return out


def cpu_baseline(cfg, inp, Xh, layer, prerouted, routing):
    """The fp64 oracle, as it stands, timed on the host cores on a bounded sample: the
    first Ts tokens of the same workload (tokens are independent in the forward, so its Y
    and dX rows are also a parity check of the GPU result, asserted to the tolerance of the dtype)."""
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
    tol = 2e-2 if cfg.dtype == "bf16" else 1e-5
    assert err_y <= tol and err_dx <= tol, "GPU result off the oracle: Y %.3e dX %.3e (tolerance %.1e)" % (err_y, err_dx, tol)
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    return {"value": round(Ts / dt, 1), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": "first %d of %d tokens, full fwd+bwd in numpy fp64 (%.1f s)" % (Ts, cfg.T, dt),
            "host_cores_available": len(os.sched_getaffinity(0)),
            "parity_on_sample": {"Y": err_y, "dX": err_dx, "tolerance": tol}}


if __name__ == "__main__":
    main()
