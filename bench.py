#!/usr/bin/env python3
"""Benchmark of the MONA optimizer step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

One "step" is one mona_step over every matrix of the workload: the fused elementwise state
kernel + norm, T = 5 Newton-Schulz iterations as grouped bf16 MFMA products, and the update
fused into the last product.  Inputs (bf16 parameters, fp32 gradients from the seeded AR(1)
generator) are resident in HBM before the timed region; a ring of gradient sets is cycled so
that consecutive steps see different gradients.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_F32_MFMA_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def cpu_baseline(workload, hp, budget_s: float = 30.0):
    """Time the float64 oracle (as it stands) on a bounded sample of the workload's matrices
    and extrapolate to a whole step by the flop count of the oracle's literal formulation."""
    import numpy as np
    import torch

    from oracle import mona_oracle as orc
    from paper_2605_26842_amd import workloads as wl

    ohp = orc.OracleHParams(hp.lr, hp.momentum, hp.beta_a, hp.alpha, hp.weight_decay, hp.ns_steps,
                            hp.ns_a, hp.ns_b, hp.ns_c, hp.ns_eps, hp.gamma_coeff).f32()

    def literal_flops(m, n):
        # S = X X^T (m x m), S X, S (S X): 3 products of 2 m^2 n flop per iteration
        return ohp.ns_steps * 3 * 2.0 * m * m * n + 20.0 * m * n

    shapes = workload.shapes()
    classes = {}
    for s in shapes:
        classes[s] = classes.get(s, 0) + 1
    # cheapest classes first; stop when the budget is used
    order = sorted(classes, key=lambda s: literal_flops(*s))
    measured, spent = {}, 0.0
    rate = None  # flop/s seen so far
    for s in order:
        est = literal_flops(*s) / rate if rate else 0.0
        if measured and spent + est > budget_s:
            continue
        w = wl.draw_weight(s, 123, torch.float32).double().numpy()
        g = wl.GradientStream(s, 456).next().double().numpy()
        o = orc.MonaOracle(s)
        t0 = time.perf_counter()
        o.step(w, g, ohp)
        dt = time.perf_counter() - t0
        measured[s] = dt
        spent += dt
        rate = literal_flops(*s) / dt
    total = 0.0
    for s, cnt in classes.items():
        if s in measured:
            total += cnt * measured[s]
        else:
            total += cnt * literal_flops(*s) / rate
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    return {
        "value": 1.0 / total, "unit": "steps/s", "cores": int(threads), "kind": "oracle",
        "sample": ("one float64 oracle step on one matrix of each of the shape classes "
                   f"{sorted(measured)} ({spent:.1f} s measured), whole-workload time "
                   f"({total:.1f} s/step) extrapolated by matrix count and, for unmeasured classes, by flop count"),
        "seconds_per_step_extrapolated": total,
    }


def n_elem_bytes_w(workload) -> int:
    """Bytes of all parameters of the workload."""
    import torch
    return workload.num_elements() * (2 if workload.w_dtype == torch.bfloat16 else 4)


def bench_adamw(args) -> int:
    """The AdamW step of the non-matrix parameters (its own JSON line; not part of the headline metric)."""
    import numpy as np
    import torch

    from paper_2605_26842_amd import binding as B
    from paper_2605_26842_amd import workloads as wl

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    name = args.adamw
    shapes = wl.VECTOR_WORKLOADS[name]
    params, ring = wl.draw_vector_inputs(shapes, 1, torch.bfloat16, torch.float32, dev, steps=2)
    opt = B.AdamWOptimizer(params)
    hp = B.mona_adamw_hparams(1e-3, 0.9, 0.95, 1e-8, 0.1)
    n_elem = sum(int(np.prod(s)) for s in shapes)
    nbytes = n_elem * (4 + 4 + 4 + 2 + 4 + 4 + 2)     # read g, m, v, w; write m, v, w
    k = 0
    for _ in range(args.warmup):
        opt.step(ring[k % 2], hp); k += 1
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()       # the step is enqueued on torch's current stream, the one these events see
    for _ in range(args.steps):
        opt.step(ring[k % 2], hp); k += 1
    e1.record()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_ev = e0.elapsed_time(e1) / args.steps
    out = {
        "metric": "AdamW steps/s (non-matrix parameters)", "value": 1e3 / ms, "unit": "steps/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": name, "tensors": len(shapes), "elements": n_elem, "param_dtype": "bfloat16",
                   "grad_dtype": "f32"},
        "roofline": {"kernel": "adamw_kernel<float, bf16>", "bound": "hbm", "achieved": nbytes / (ms_ev * 1e-3) / 1e9,
                     "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": nbytes / (ms_ev * 1e-3) / 1e9 / PEAK_HBM_GBS,
                     "traffic": None, "bytes_per_step": nbytes, "ms_per_step": ms_ev},
    }
    if not args.no_cpu_baseline:
        from oracle import adamw_oracle as ao
        n = 1 << 24
        w = np.random.default_rng(0).standard_normal(n)
        g = np.random.default_rng(1).standard_normal(n) * 1e-3
        o = ao.AdamWOracle((n,))
        t0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t0 < 10.0:
            w = o.step(w, g, ao.AdamWHParams())
            reps += 1
        dt = (time.perf_counter() - t0) / reps
        out["cpu_baseline"] = {"value": 1.0 / (dt * n_elem / n), "unit": "steps/s", "cores": 1, "kind": "oracle",
                               "sample": f"float64 oracle step on {n} elements, {reps} repetitions, scaled by element count"}
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="moe_layer_h4096_e128")
    ap.add_argument("--ns-precision", type=int, default=0)
    ap.add_argument("--state-dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--accel-form", default="two-buffer", choices=["two-buffer", "one-buffer", "caller-slot"],
                    help="two-buffer: G_{k-1} and A stored as Alg. 1 writes it; one-buffer: no stored G_{k-1} "
                         "(22 instead of 30 bytes per element in the elementwise pass); caller-slot: G_{k-1} "
                         "lives in arrays the caller keeps (Sec. 6.3's streaming form: same traffic, less state)")
    ap.add_argument("--g-dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--grad-ring", type=int, default=2)
    ap.add_argument("--muon-only", action="store_true",
                    help="plain Muon step (acceleration buffers untouched): the baseline of the paper's overhead figure")
    ap.add_argument("--zero-gradients", action="store_true",
                    help="all-zero gradients: the same launches and instruction stream on operands that do not "
                         "toggle (an experiment on the power limit, not a benchmark)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--per-launch", action="store_true", help="also print per-launch timings to stderr")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB elementwise copy (negation; a reference kernel of known traffic for "
                         "scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--ns-steps", type=int, default=5, help="Newton-Schulz iterations T (the paper's 5)")
    ap.add_argument("--ns-schedule", default="auto", choices=["auto", "literal", "fused", "pairs"],
                    help="layout of the Newton-Schulz iterations as products: literal = Gram, poly, apply per "
                         "iteration; fused = chunks of three then two iterations advanced on the p x p side; pairs = chunks of "
                         "two; auto = the library's choice per shape group")
    ap.add_argument("--overlap", default="off", choices=["off", "late-group"],
                    help="late-group: the elementwise pass of the largest shape group runs beside the products of the "
                         "other groups on a quarter of the CUs; off (the library's default): one elementwise pass "
                         "over everything first")
    ap.add_argument("--streams", type=int, default=0,
                    help="streams the shape groups' launch chains are spread over (0 = library default, 1 = one)")
    ap.add_argument("--graph", action="store_true",
                    help="record one step into a HIP graph and time replays of it (for launch-bound small "
                         "workloads; uses one static gradient set)")
    ap.add_argument("--adamw", default=None, metavar="VECTOR_WORKLOAD",
                    help="instead of the MONA step, time the AdamW step of a set of non-matrix parameters "
                         "(embeddings_h4096_v128k or small_vectors) and print its own JSON line")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import torch

    from paper_2605_26842_amd import binding as B
    from paper_2605_26842_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    if args.adamw:
        return bench_adamw(args)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    # everything below runs on one stream of its own (default priority), not on the null stream: the library
    # can then run part of the elementwise pass beside the products (the null stream would serialise them)
    torch.cuda.set_stream(torch.cuda.Stream(dev))
    workload = wl.WORKLOADS[args.workload]
    widx = list(wl.WORKLOADS).index(args.workload)
    hp = wl.HParams(flags=B.MONA_FLAG_MUON_ONLY if args.muon_only else 0, ns_steps=args.ns_steps)
    shapes = workload.shapes()
    g_dtype = torch.float32 if args.g_dtype == "f32" else torch.bfloat16
    state_dtype = torch.float32 if args.state_dtype == "f32" else torch.bfloat16

    # inputs, resident before timing
    weights = [wl.draw_weight(s, wl.matrix_seed(widx, i), workload.w_dtype, dev) for i, s in enumerate(shapes)]
    ring = []
    streams = None
    for r in range(1 if args.graph else max(1, args.grad_ring)):
        if streams is None:
            # one generator state per shape class keeps the host loop short; each matrix still
            # gets its own draw
            streams = [wl.GradientStream(s, wl.matrix_seed(widx, i), dev) for i, s in enumerate(shapes)]
        ring.append([st.next().to(g_dtype) for st in streams])
    if args.zero_gradients:
        for gs in ring:
            for g in gs:
                g.zero_()
    del streams
    accel_form = {"two-buffer": B.MONA_ACCEL_TWO_BUFFER, "one-buffer": B.MONA_ACCEL_ONE_BUFFER,
                  "caller-slot": B.MONA_ACCEL_CALLER_SLOT}[args.accel_form]
    slots = None
    if accel_form == B.MONA_ACCEL_CALLER_SLOT:
        slots = [torch.zeros(s, dtype=state_dtype, device=dev) for s in shapes]
    opt = B.MonaOptimizer(weights, ns_precision=args.ns_precision, state_dtype=state_dtype, g_dtype=g_dtype,
                          accel_form=accel_form, max_streams=args.streams,
                          ns_schedule={"auto": 0, "literal": 1, "fused": 2, "pairs": 3}[args.ns_schedule],
                          overlap={"off": 0, "late-group": 1}[args.overlap])
    hpc = B.make_hparams(hp)
    plan = opt.plan_info(hp.ns_steps)
    torch.cuda.synchronize()

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        torch.neg(src, out=dst)   # reads 1 GiB, writes 1 GiB, in a kernel nothing else here launches
        torch.cuda.synchronize()
        del src, dst

    k = 0
    for _ in range(args.warmup):
        opt.step(ring[k % len(ring)], hpc, slots)
        k += 1
    torch.cuda.synchronize()

    graph = None
    if args.graph:
        opt.step(ring[0], hpc, slots)      # the pointer table now names ring[0]: the capture holds launches only
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            opt.step(ring[0], hpc, slots)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps

    # timed region: exactly --steps steps; phase times come from HIP events that mona_step
    # records on the stream it launches on
    opt.set_profiling(1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        opt.step(ring[k % len(ring)], hpc, slots)
        k += 1
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    eager_ms = ms_per_step
    if graph is not None:
        ms_per_step = graph_ms      # the phase split below still comes from eager, profiled steps
    # phase split: the HIP events the library recorded, on the stream it launched on, around the
    # phases of these very steps (it keeps the marks of the last 32 profiled steps)
    (ew_ms, ns_ms, upd_ms, step_ms_events), n_phase = opt.mean_step_times()

    # The same phases one after the other on one stream (level 2 also times every launch): in the timed steps
    # the elementwise pass of the largest shape group may run beside the products of the other groups, on a
    # quarter of the CUs, and is then hidden inside the Newton-Schulz interval above
    opt.set_profiling(2)
    for _ in range(3):
        opt.step(ring[k % len(ring)], hpc, slots)
        k += 1
    (ew_serial_ms, ns_serial_ms, _, step_serial_ms), _ = opt.mean_step_times()
    launches = opt.last_step_launches()
    # Step (c), the parameter update: it rides in the epilogue of each group's last apply launch.  Its HBM
    # traffic is W read + W written; its cost is what those launches take beyond an apply of the same group
    # that carries no update.
    fused_upd_ms = plain_ms = 0.0
    groups_seen = set()
    for r in launches:
        if r["kind"] == 2 and r["iter"] == hp.ns_steps - 1:
            others = [q["ms"] for q in launches if q["kind"] == 2 and q["group"] == r["group"] and q["iter"] != r["iter"]]
            if others:
                fused_upd_ms += r["ms"]
                plain_ms += sum(others) / len(others)
                groups_seen.add(r["group"])
    w_bytes = 2 * n_elem_bytes_w(workload)
    if args.per_launch:
        kinds = {0: "gram", 1: "poly", 2: "apply", 3: "sym"}
        for r in launches:
            tf = r["flops"] / (r["ms"] * 1e-3) / 1e12 if r["ms"] > 0 else 0.0
            print(f"[launch] {kinds[r['kind']]:5s} {r['m']}x{r['n']} x{r['count']} iter {r['iter']} tile {r['tile']}: "
                  f"{r['ms']:.3f} ms  {tf:.1f} TFLOP/s issued", file=sys.stderr)
    opt.set_profiling(1)

    n_elem = workload.num_elements()
    flops_sym = workload.ns_flops_symmetric(hp.ns_steps)
    flops_dense = workload.ns_flops_dense(hp.ns_steps)
    peak = PEAK_F32_MFMA_TFLOPS if args.ns_precision == 1 else PEAK_BF16_TFLOPS
    ns_tflops = flops_sym / (ns_ms * 1e-3) / 1e12 if ns_ms > 0 else 0.0
    ew_bytes = plan["elementwise_bytes"]
    if args.muon_only:   # G and M read, M and the working copy written
        ew_bytes = n_elem * ((4 if args.g_dtype == "f32" else 2) + 4 + 4 + 2)
    ew_gbs = ew_bytes / (ew_serial_ms * 1e-3) / 1e9 if ew_serial_ms > 0 else 0.0

    # HBM bytes per launch measured with rocprofv3 counters (a committed summary, not measured here)
    traffic_ns = traffic_ew = traffic_source = None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{args.workload}.json")
    if os.path.exists(tpath) and args.ns_precision == 0 and args.g_dtype == "f32" and args.state_dtype == "f32" \
            and not args.muon_only and args.accel_form == "two-buffer":
        with open(tpath) as f:
            tj = json.load(f)
        # the figures belong to the launch plan they were measured on: dropped when the plan has changed since
        if tj.get("ns_launches_per_step") == plan["ns_launches"]:
            traffic_ns = tj.get("ns_gemm_bytes_per_launch")
        traffic_ew = tj.get("state_update_bytes_per_launch")
        traffic_source = f"profiles/traffic_{args.workload}.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this " \
                         "command, committed; not measured in this run)"

    out = {
        "metric": "MONA optimizer steps/s",
        "value": 1e3 / ms_per_step,
        "unit": "steps/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if args.ns_precision == 0 else "f32",
        "data": "synthetic",
        "config": {
            "workload": args.workload, "matrices": len(shapes), "elements": n_elem,
            "param_dtype": str(workload.w_dtype).replace("torch.", ""), "grad_dtype": args.g_dtype,
            "state_dtype": args.state_dtype, "accel_form": args.accel_form, "ns_steps": hp.ns_steps, "ns_precision": args.ns_precision,
            "grad_ring": len(ring), "optimizer": "muon" if args.muon_only else "mona",
            "launch": "hip graph replay" if graph is not None else "eager", "streams": args.streams,
            "ns_schedule": args.ns_schedule, "overlap": args.overlap, "zero_gradients": bool(args.zero_gradients),
        },
        "roofline": {
            "kernel": "ns_gemm (grouped Newton-Schulz products, %d launches/step)" % plan["ns_launches"],
            "bound": "mfma", "achieved": ns_tflops, "peak": peak, "unit": "TFLOP/s",
            "frac": ns_tflops / peak,
            "traffic": traffic_ns,
            "traffic_source": traffic_source,
            "flops_per_step_algorithmic": flops_sym,
            "flops_per_step_issued": plan["ns_flops_issued"],
            "flops_per_step_dense_equivalent": flops_dense,
            "ms_per_step": ns_ms,
            "avg_launch_ms": ns_ms / max(plan["ns_launches"], 1),
            "ms_per_step_phases_in_a_row": ns_serial_ms,
            "elementwise": {"bound": "hbm", "achieved": ew_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                            "frac": ew_gbs / PEAK_HBM_GBS},
        },
        "elementwise": {
            "kernel": "state_update + norm_finalize", "bound": "hbm", "achieved": ew_gbs, "peak": PEAK_HBM_GBS,
            "unit": "GB/s", "frac": ew_gbs / PEAK_HBM_GBS, "bytes_per_step": ew_bytes, "ms_per_step": ew_serial_ms,
            "traffic": traffic_ew,
            "measured": "3 steps after the timed ones with the phases one after the other on the launch stream "
                        "(in the timed steps part of this pass may run beside the products on a quarter of the CUs)",
        },
        "update": {
            "kernel": "last apply launch of every shape group (Eq. muon_update fused into its epilogue)",
            "bound": "hbm", "bytes_per_step": w_bytes,
            "ms_update_launches": fused_upd_ms, "ms_same_launches_without_update": plain_ms,
            "ms_added_by_update": fused_upd_ms - plain_ms,
            "achieved_over_the_launches": w_bytes / (fused_upd_ms * 1e-3) / 1e9 if fused_upd_ms > 0 else None,
            "achieved_over_the_added_time": w_bytes / ((fused_upd_ms - plain_ms) * 1e-3) / 1e9 if fused_upd_ms > plain_ms else None,
            "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "note": "the launches are bound by the matrix units; the parameter traffic hides behind their products, "
                    "so over the added time alone it can exceed the HBM peak",
        },
        "phases_ms": {"elementwise_before_products": ew_ms, "newton_schulz": ns_ms, "separate_update": upd_ms,
                      "step_events": step_ms_events, "steps_averaged": n_phase,
                      "in_a_row": {"elementwise": ew_serial_ms, "newton_schulz": ns_serial_ms, "step": step_serial_ms}},
        "ns_tflops_dense_equivalent": flops_dense / (ns_ms * 1e-3) / 1e12 if ns_ms > 0 else 0.0,
        "ns_tflops_issued": plan["ns_flops_issued"] / (ns_ms * 1e-3) / 1e12 if ns_ms > 0 else 0.0,
    }
    if graph is not None:
        out["eager_ms_per_step"] = eager_ms
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(workload, hp)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
