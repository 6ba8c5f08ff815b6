#!/usr/bin/env python3
"""Benchmark of the rotated W8A8 linear path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input: for every
linear of a DiT-XL/2-shaped block (qkv, proj, fc1, fc2) at 4096 tokens, look up the sampling
step's group, rotate + quantise the bf16 activations (trdq_rotate_quant) and run the int8
product with the dequantising epilogue (trdq_qgemm) against that group's prepared weights.
Inputs, diagonals and prepared weights are resident in HBM before the timed region.

Prints ONE JSON line: whole-job int8 TOP/s (2*M*K*N summed over the four linears per step,
divided by wall time), plus `roofline` for the dominant kernel (qgemm, int8 MFMA bound; its
launch durations are measured with events on the launch stream inside the timed region) and
`cpu_baseline` (the CPU oracle timed on a bounded sample of the same workload).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0      # MI355X dense int8, published
HBM_PEAK_GBS = 8000.0             # MI355X HBM3E, published


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=1, help="workload config id (1 = the metric's)")
    ap.add_argument("--fused", action="store_true", help="use the fused kernel instead of rotate_quant + qgemm")
    ap.add_argument("--no-events", action="store_true", help="no per-kernel events in the timed region")
    ap.add_argument("--event-every", type=int, default=0,
                    help="bracket the kernels with events on every n-th timed step (keeps the probe effect small); "
                         "0 = max(1, steps // 10), so that at least ten launches stand behind every kernel figure")
    ap.add_argument("--no-tiled", action="store_true",
                    help="row-major activation codes for every linear (trdq_rotate_quant + trdq_qgemm), also where "
                         "the library prefers the block-tiled pair")
    ap.add_argument("--graph", action="store_true",
                    help="replay one captured HIP graph per step instead of launching every kernel from the host "
                         "(same kernels; measured to make no difference here: the step is GPU-bound, and the "
                         "profiler's kernel trace does not list kernels launched from a graph)")
    ap.add_argument("--rpr", action="store_true",
                    help="the full transform of Eq. 9 (rotation, zigzag permutation, rotation) instead of one rotation")
    ap.add_argument("--asym", action="store_true",
                    help="asymmetric per-token activation codes (zero point, Eq. 1-3) instead of symmetric ones; W8 only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-measured-peaks", action="store_true",
                    help="skip the yardstick kernels that give roofline.measured_peak")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="CPU work budget of the oracle's timed sample")
    ap.add_argument("--variant", type=int, default=-1, help="qgemm tile variant override")
    ap.add_argument("--groups", type=int, default=0, help="limit the number of groups prepared (0 = all)")
    ap.add_argument("--no-warm", action="store_true",
                    help="plain rotate_quant: do not read the following product's weights on the way")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one 256 MiB device copy (a kernel of known traffic, to calibrate counters)")
    return ap.parse_args()


def cpu_baseline(cfg, wl, budget_s):
    """The oracle, as it stands, on the same workload: whole groups (all tokens of every linear
    of the block) until about `budget_s` seconds of CPU work are spent."""
    from oracle import trdq_oracle as o
    o.lib()
    group = None if cfg.wbits[0] == 8 else 128
    ops, tokens, spent, groups = 0, 0, 0.0, 0
    for g in range(cfg.n_groups):
        step = next(s for s in range(cfg.n_steps) if wl.draw_group(cfg, s) == g)
        prepared = {}
        for kind in cfg.kinds:                       # untimed: inputs and the offline weight side
            d = wl.make_diag(cfg, kind, g)
            prepared[kind] = (wl.make_x(cfg, kind, step), d, wl.make_bias(cfg, kind),
                              o.prepare_weights(wl.make_w(cfg, kind), d, 128, cfg.wbits[0]))
        t0 = time.perf_counter()
        for kind in cfg.kinds:
            Xb, d, bias, (Wq, sw) = prepared[kind]
            Xq, sx = o.rotate_quant(Xb, d)
            acc = o.igemm(Xq, Wq, group)
            o.dequant(acc, sx, sw, bias)
            K, N = wl.LAYER_SHAPES[kind]
            ops += 2 * cfg.M * K * N
        spent += time.perf_counter() - t0
        tokens += cfg.M
        groups += 1
        if spent >= budget_s:
            break
    return {"value": ops / spent / 1e12, "unit": "TOP/s", "cores": o.threads(), "kind": "oracle",
            "tokens_per_s": tokens / spent,
            "sample": f"{groups} of {cfg.n_groups} groups x {cfg.M} tokens x {len(cfg.kinds)} linears "
                      f"(rotate+quantise, int32 product, dequant; weights prepared beforehand, untimed), "
                      f"{spent:.1f} s of CPU work"}


def committed_traffic(workload, config):
    """HBM bytes per qgemm launch from the committed counter summary of this workload, or None.

    The figure comes from the two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) of this same
    command, scaled by the copy-kernel calibration; the summary file states the commands."""
    path = os.path.join(ROOT, "profiles", f"bench_config{config}_{workload}.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


class HipEvent:
    """A timing event without the system-scope fence that a default event carries: a default
    event makes the device flush its caches for the host before the next kernel may start, about
    5 us per event here, which would land inside every bracketed interval."""
    _hip = None
    DISABLE_SYSTEM_FENCE = 0x20000000        # hipEventDisableSystemFence

    def __init__(self):
        import ctypes
        if HipEvent._hip is None:
            hip = ctypes.CDLL("libamdhip64.so")
            hip.hipEventCreateWithFlags.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint]
            hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
            hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
            hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
            HipEvent._hip = hip
        self.h = ctypes.c_void_p()
        rc = HipEvent._hip.hipEventCreateWithFlags(ctypes.byref(self.h), HipEvent.DISABLE_SYSTEM_FENCE)
        assert rc == 0, f"hipEventCreateWithFlags: {rc}"

    def record(self, stream):
        rc = HipEvent._hip.hipEventRecord(self.h, stream.cuda_stream)
        assert rc == 0, f"hipEventRecord: {rc}"

    def elapsed_time(self, other):
        import ctypes
        ms = ctypes.c_float()
        rc = HipEvent._hip.hipEventElapsedTime(ctypes.byref(ms), self.h, other.h)
        assert rc == 0, f"hipEventElapsedTime: {rc}"
        return ms.value


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (tokens are independent rows; more GPUs would "
              "shard them with replicated weights) -- run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2503_06564_amd import trdq, workloads as wl

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    trdq.lib()
    dev = torch.device("cuda:0")
    cfg = wl.CONFIGS[args.config]
    wbits = cfg.wbits[0]
    M = cfg.M
    n_groups = cfg.n_groups if args.groups <= 0 else min(args.groups, cfg.n_groups)
    trdq.qgemm_set_variant(args.variant)

    table = trdq.Table(cfg.n_steps, cfg.n_groups)
    # everything runs on one side stream (default priority): graph capture needs a non-default stream
    stream = torch.cuda.Stream()
    torch.cuda.set_stream(stream)

    # ---- resident state: per kind and group, activations, diagonal, prepared weights ----------
    X, D, Wh, B, Y, Xq, SX, P, ZC = {}, {}, {}, {}, {}, {}, {}, {}, {}
    for kind in cfg.kinds:
        K, N = wl.LAYER_SHAPES[kind]
        Wd = torch.from_numpy(wl.make_w(cfg, kind)).to(dev)
        B[kind] = torch.from_numpy(wl.make_bias(cfg, kind)).to(dev)
        Y[kind] = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        Xq[kind] = torch.empty((M, K), dtype=torch.int8, device=dev)
        SX[kind] = torch.empty((M,), dtype=torch.float32, device=dev)
        ZC[kind] = torch.empty((M,), dtype=torch.int32, device=dev)
        for g in range(n_groups):
            step_of_g = next(s for s in range(cfg.n_steps) if wl.draw_group(cfg, s) == g)
            xb = wl.make_x(cfg, kind, step_of_g)
            X[kind, g] = torch.from_numpy(xb.view(np.int16)).to(dev).view(torch.bfloat16)
            D[kind, g] = torch.from_numpy(wl.make_diag(cfg, kind, g)).to(dev)
            if args.rpr:
                # zigzag permutation from the per-channel absmax of this group's once-rotated activations
                mag = torch.empty((K,), dtype=torch.float32, device=dev)
                trdq.channel_absmax(X[kind, g], D[kind, g], mag, rotate=True)
                P[kind, g] = torch.from_numpy(trdq.zigzag_permutation(mag.cpu().numpy())).to(dev)
                Wh[kind, g] = trdq.prepare_weights_rpr(Wd, D[kind, g], P[kind, g], wbits=wbits)
            else:
                Wh[kind, g] = trdq.prepare_weights(Wd, D[kind, g], wbits=wbits)
        del Wd
    torch.cuda.synchronize()

    ops_step = sum(2 * M * K * N for K, N in (wl.LAYER_SHAPES[k] for k in cfg.kinds))
    gemm_ops = {k: 2 * M * wl.LAYER_SHAPES[k][0] * wl.LAYER_SHAPES[k][1] for k in cfg.kinds}
    rq_bytes = {k: M * (3 * wl.LAYER_SHAPES[k][0] + 4) for k in cfg.kinds}

    use_events = not args.no_events

    # one pre-marshalled C call per launch (the binding converts the arguments once)
    calls = {}
    tiled_kinds = set()
    for g in range(n_groups):
        for kind in cfg.kinds:
            if args.fused:
                calls[g, kind] = (trdq.bind_linear_fused(X[kind, g], D[kind, g], Wh[kind, g], Y[kind],
                                                         bias=B[kind], stream=stream),)
            elif args.asym:
                calls[g, kind] = (trdq.bind_rotate_quant_asym(X[kind, g], D[kind, g], Xq[kind], SX[kind], ZC[kind],
                                                              stream=stream,
                                                              warm=None if args.no_warm else Wh[kind, g]),
                                  trdq.bind_qgemm_asym(Wh[kind, g], Xq[kind], SX[kind], ZC[kind], Y[kind],
                                                       bias=B[kind], stream=stream))
            elif args.rpr:
                calls[g, kind] = (trdq.bind_rotate_quant_rpr(X[kind, g], D[kind, g], P[kind, g], Xq[kind], SX[kind],
                                                             stream=stream,
                                                             warm=None if args.no_warm else Wh[kind, g]),
                                  trdq.bind_qgemm(Wh[kind, g], Xq[kind], SX[kind], Y[kind], bias=B[kind],
                                                  stream=stream))
            elif not args.no_tiled and args.variant < 0 and trdq.qgemm_tiled_preferred(Wh[kind, g], M):
                # the shapes for which the library itself (trdq_layer_forward) takes the block-tiled pair;
                # Xq[kind] holds M * K bytes in either form (M is a multiple of 128 here)
                tiled_kinds.add(kind)
                calls[g, kind] = (trdq.bind_rotate_quant_tiled(X[kind, g], D[kind, g], Xq[kind], SX[kind],
                                                               stream=stream,
                                                               warm=None if args.no_warm else Wh[kind, g]),
                                  trdq.bind_qgemm_tiled(Wh[kind, g], Xq[kind], SX[kind], Y[kind], bias=B[kind],
                                                        stream=stream))
            else:
                calls[g, kind] = (trdq.bind_rotate_quant(X[kind, g], D[kind, g], Xq[kind], SX[kind], stream=stream,
                                                         warm=None if args.no_warm else Wh[kind, g]),
                                  trdq.bind_qgemm(Wh[kind, g], Xq[kind], SX[kind], Y[kind], bias=B[kind],
                                                  stream=stream))
    n_ev = len(cfg.kinds) * (2 if args.fused else 3)
    every = args.event_every if args.event_every > 0 else max(1, args.steps // 10)
    events = {st: [HipEvent() for _ in range(n_ev)]
              for st in range(0, args.steps, every)} if use_events else {}
    ev = []     # (name, kind, start, end)

    def run_step(step, record):
        g = table.lookup(step % cfg.n_steps) % n_groups
        evs = events.get(step) if record else None
        record = evs is not None
        i = 0
        for kind in cfg.kinds:
            fns = calls[g, kind]
            if record:
                evs[i].record(stream)
            for j, fn in enumerate(fns):
                fn()
                if record:
                    evs[i + j + 1].record(stream)
            if record:
                if args.fused:
                    ev.append(("fused", kind, evs[i], evs[i + 1]))
                else:
                    ev.append(("rotate_quant", kind, evs[i], evs[i + 1]))
                    ev.append(("qgemm", kind, evs[i + 1], evs[i + 2]))
                i += len(fns) + 1
        if record:
            ev.append(("step", "-", evs[0], evs[i - 1]))       # the whole step, first to last event

    for s in range(args.warmup):
        run_step(s, False)
    torch.cuda.synchronize()

    # One captured graph per time-step group: the step's launches (8 kernels) replayed as a unit, so
    # the host's per-launch cost does not throttle kernels of 10-30 us.  Steps that carry events are
    # launched from the host as before (same kernels, same arguments).
    graphs = {}
    if args.graph:
        for g in range(n_groups):
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr, stream=stream):
                for kind in cfg.kinds:
                    for fn in calls[g, kind]:
                        fn()
            graphs[g] = gr
        torch.cuda.set_stream(stream)
        for g in range(n_groups):      # one untimed replay each
            graphs[g].replay()
        torch.cuda.synchronize()

    def timed_step(step):
        if graphs and step not in events:
            graphs[table.lookup(step % cfg.n_steps) % n_groups].replay()
        else:
            run_step(step, use_events)

    t0 = time.perf_counter()
    for s in range(args.steps):
        timed_step(s)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    if args.copy_probe:
        # a kernel of known traffic for the counter runs: 256 MiB read + 256 MiB written
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    ms_per_step = dt / args.steps * 1e3
    value = ops_step * args.steps / dt / 1e12
    out = {
        "metric": "int8 TOP/s of the rotated W8A8 linears of one DiT-XL/2-shaped block "
                  "(rotate_quant + qgemm per linear, 2*M*K*N ops)",
        "value": value, "unit": "TOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8" if wbits == 8 else "int8xint4", "data": "synthetic",
        "tokens_per_s": M * args.steps / dt,
        "config": {"workload": cfg.name, "tokens": M, "layers": list(cfg.kinds), "groups": n_groups,
                   "path": "fused" if args.fused else ("rotate_quant_rpr+qgemm" if args.rpr else ("rotate_quant_asym+qgemm_asym" if args.asym else "rotate_quant+qgemm")), "wbits": wbits,
                   "block_tiled_codes": sorted(tiled_kinds),
                   "launch": "hip graph per step" if graphs else "host launches"},
    }

    if use_events and ev:
        per = {}
        for name, kind, a, b in ev:
            per.setdefault((name, kind), []).append(a.elapsed_time(b) * 1e-3)
        kern = {}
        # What a bracket adds to its kernel (the device's handling of the event records; it differs
        # with and without a profiler attached) is calibrated from the run itself: the steps
        # without events run back to back, so their average length is the sum of their kernels'
        # durations; the brackets of an evented step add up to more, and the excess is spread
        # evenly over its launches.
        spans = per.pop(("step", "-"))
        n_plain = args.steps - len(spans)
        t_plain = (dt - sum(spans)) / n_plain if n_plain > 0 else 0.0
        n_kernels = sum(len(calls[0, kind]) for kind in cfg.kinds)
        bracket_sum = sum(sum(ts) for ts in per.values()) / len(spans)
        ev_cost = max(0.0, (bracket_sum - t_plain) / n_kernels) if n_plain > 0 else 0.0
        for (name, kind), ts in per.items():
            per[name, kind] = ts = [max(t - ev_cost, 0.0) for t in ts]
        for (name, kind), ts in per.items():
            avg = sum(ts) / len(ts)
            entry = {"avg_us": avg * 1e6, "median_us": sorted(ts)[len(ts) // 2] * 1e6, "launches": len(ts)}
            if avg <= 0.0:                 # a bracket no longer than its calibrated cost (profiler attached): no rate
                kern[f"{name}:{kind}"] = entry
                continue
            if name in ("qgemm", "fused"):
                entry["tops"] = gemm_ops[kind] / avg / 1e12
                entry["frac_int8_peak"] = entry["tops"] / INT8_MFMA_PEAK_TOPS
            if name == "rotate_quant":
                entry["gbs"] = rq_bytes[kind] / avg / 1e9
                entry["frac_hbm_peak"] = entry["gbs"] / HBM_PEAK_GBS
            kern[f"{name}:{kind}"] = entry
        out["kernels"] = kern
        dom = "fused" if args.fused else "qgemm"
        tot_t = sum(sum(ts) for (name, _), ts in per.items() if name == dom)
        n_launch = sum(len(ts) for (name, _), ts in per.items() if name == dom)
        tot_ops = sum(gemm_ops[kind] * len(ts) for (name, kind), ts in per.items() if name == dom)
        achieved = tot_ops / tot_t / 1e12 if tot_t > 0 else 0.0
        out["roofline"] = {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": INT8_MFMA_PEAK_TOPS,
                           "unit": "TOP/s", "frac": achieved / INT8_MFMA_PEAK_TOPS, "traffic": None,
                           "avg_launch_us": tot_t / max(n_launch, 1) * 1e6, "launches": n_launch,
                           "event_cost_us": ev_cost * 1e6,
                           "timed_on": f"every {every}th of the {args.steps} timed steps (launched from the host, "
                                       "the others replay a captured graph if --graph), events on the launch stream; "
                                       "event_cost_us = (sum of an evented step's brackets - average length of "
                                       "a step without events) / launches per step is subtracted from every bracket",
                           "ops_per_launch": tot_ops / max(n_launch, 1)}
        if not args.fused and sum(sum(ts) for (name, _), ts in per.items() if name == "rotate_quant") > 0:
            rq_t = sum(sum(ts) for (name, _), ts in per.items() if name == "rotate_quant")
            rq_b = sum(rq_bytes[kind] * len(ts) for (name, kind), ts in per.items() if name == "rotate_quant")
            out["roofline_rotate_quant"] = {"bound": "hbm", "achieved": rq_b / rq_t / 1e9, "peak": HBM_PEAK_GBS,
                                            "unit": "GB/s", "frac": rq_b / rq_t / 1e9 / HBM_PEAK_GBS,
                                            "traffic": None}

    if "roofline" in out:
        # HBM bytes per launch are not measured by this run: they come from the committed counter summary
        # of the same command (two rocprofv3 --pmc runs), or stay null when there is none
        out["roofline"]["traffic"] = committed_traffic(cfg.name, args.config)
        out["roofline"]["traffic_source"] = (f"profiles/bench_config{args.config}_{cfg.name}.txt (rocprofv3 --pmc FETCH_SIZE / "
                                             "WRITE_SIZE of this command, committed; not measured in this run)"
                                             if out["roofline"]["traffic"] is not None else None)
        if not args.no_measured_peaks:
            # after the timed region: the chip's own ceilings for the two bounding operations
            # (register-only int8 matrix issue; a pass of 2 bytes read + 1 written per element)
            from paper_2503_06564_amd.microbench import measure_peaks
            shapes = sorted({(M, wl.LAYER_SHAPES[kind][0]) for kind in cfg.kinds})
            pk = measure_peaks(dev, quick=True, stream_sizes=shapes)
            out["roofline"]["measured_peak"] = pk["mfma_i8_tops"]
            out["roofline"]["frac_of_measured"] = out["roofline"]["achieved"] / pk["mfma_i8_tops"]
            # the same register-only loop on random operand bytes (the clock drops with the pipes' power draw)
            out["roofline"]["measured_peak_random_operands"] = pk["mfma_i8_data_tops"]
            out["roofline"]["frac_of_measured_random_operands"] = out["roofline"]["achieved"] / pk["mfma_i8_data_tops"]
            if "roofline_rotate_quant" in out:
                # the same mix of shapes as the step's rotate_quant launches, streamed without arithmetic
                rq = out["roofline_rotate_quant"]
                t_y = sum(pk["stream_us"][f"{M}x{wl.LAYER_SHAPES[kind][0]}"] for kind in cfg.kinds) * 1e-6
                b_y = sum(3.0 * M * wl.LAYER_SHAPES[kind][0] for kind in cfg.kinds)
                rq["measured_peak"] = b_y / t_y / 1e9
                rq["frac_of_measured"] = rq["achieved"] / rq["measured_peak"]

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, wl, args.cpu_seconds)

    print(json.dumps(out))


if __name__ == "__main__":
    main()
