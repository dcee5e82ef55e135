"""Benchmark: forward+backward images/s of a micro-DAG kernel on one MI355X, with the roofline fraction
of its dominant kernel and the CPU oracle timed beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload shift_residual|involution|sampled_cC_hH]
    python bench.py --workload chain_gate|chain_relu|chain_shift_residual|chain_box3|chain_softmax_c[_cC_hH]
                                                       (an FC-free fused chain at a ResNet layer shape, N=128, vs the HBM roof)
    python bench.py --workload block_64_256      (a block C_in=64 => C_out=256 composed of four shift_residual templates)
    python bench.py --workload fuzz [--seeds 100:300] [--compare]  (config 5: geometric mean over the random DAGs, chain kernels vs HBM)
    python bench.py --fc-micro                         (grouped-FC kernels of config 4, operands in cache, vs MFMA peak)
    python bench.py --infer BATCH [--workload ...]     (forward-only latency of the inference plan, not the headline)

The default run measures config 2 (`value`) and adds `per_config`: config 3 and the four shapes of config 4.

One step = one forward + one backward of the whole micro-DAG over one batch resident in HBM.  Buffer
sets are rotated so that consecutive steps do not find their operands in the 256 MB last-level cache.
Prints one JSON line.
"""
import argparse
import json
import math
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0


# HBM bytes per launch from two `rocprofv3 --pmc` runs of this file per workload (FETCH_SIZE, then WRITE_SIZE; the runtime's
# plain copy of 25 088 KiB reads FETCH_SIZE 12 557 -> units of 1.998 KiB, and WRITE_SIZE 25 088 -> KiB; the dispatches of
# a run are attributed to the launches of a step by position; commands and tables in profiles/).  The figures are valid
# only for the kernel sources they were taken on (one hash over the library's source folder), otherwise `traffic` is null.
TRAFFIC_SHA256 = "8e421938639fd978f6a91276b051d50575fb67a893047c1943244e723da8e289"
TRAFFIC_KIB = {  # workload -> launch (phase:name) -> (KiB fetched, KiB written) per launch
    'shift_residual': {'fwd:sgfc_fwd': (28773.5, 25090.9), 'bwd:sgfc_bwd': (52695.2, 25890.3), 'bwd:sgfc_dw_reduce': (3226.7, 4.0)},
    'involution': {'fwd:weight_prep': (326.0, 40.0), 'fwd:dyn_fc1_softmax': (6732.3, 882.0), 'fwd:dyn_apply': (7266.3, 6272.0), 'fwd:dyn_fc2': (6990.8, 6272.0), 'bwd:dyn_fc2_wgrad': (15871.7, 6656.0), 'bwd:dyn_fc2_dgrad': (6990.8, 6272.0), 'bwd:dyn_apply_dx_da': (20213.4, 7154.2), 'bwd:dyn_softmax_bwd': (2088.0, 1323.0), 'bwd:dyn_fc1_wgrad': (10051.7, 900.0), 'bwd:dyn_fc1_dgrad': (7235.0, 6272.0), 'bwd:wgrad_reduce': (7617.2, 68.5)},
    'sampled_c64_h56': {'fwd:weight_prep': (169.0, 44.0), 'fwd:ufc_fc1_unfold': (50562.9, 50176.0), 'fwd:ufc_mid_fwd': (101104.5, 50182.7), 'fwd:ufc_fc2': (50606.7, 50176.0), 'bwd:ufc_fc2_wgrad': (100519.2, 6272.0), 'bwd:ufc_fc2_dgrad': (50606.7, 50176.0), 'bwd:ufc_mid_bwd': (152855.0, 100352.0), 'bwd:ufc_fc1_wgrad_unfold': (105580.2, 4608.0), 'bwd:ufc_fc1_dgrad_unfold': (100704.1, 50176.0), 'bwd:wgrad_reduce': (10937.7, 104.0)},
    'sampled_c128_h28': {'fwd:weight_prep': (531.7, 104.0), 'fwd:ufc_fc1_unfold': (25631.4, 25099.4), 'fwd:ufc_mid_fwd': (50596.6, 25093.1), 'fwd:ufc_fc2': (26279.9, 25094.6), 'bwd:ufc_fc2_wgrad': (65423.1, 6656.0), 'bwd:ufc_fc2_dgrad': (26279.9, 25088.0), 'bwd:ufc_mid_bwd': (76486.0, 50176.0), 'bwd:ufc_fc1_wgrad_unfold': (60974.9, 4608.0), 'bwd:ufc_fc1_dgrad_unfold': (50697.8, 25127.5), 'bwd:wgrad_reduce': (11321.3, 416.0)},
    'sampled_c256_h14': {'fwd:weight_prep': (2214.1, 416.0), 'fwd:ufc_fc1_unfold': (13282.1, 12563.2), 'fwd:ufc_mid_fwd': (25905.1, 12871.0), 'fwd:ufc_fc2': (14591.9, 12592.0), 'bwd:ufc_fc2_wgrad': (25347.3, 8192.0), 'bwd:ufc_fc2_dgrad': (14591.8, 12592.0), 'bwd:ufc_mid_bwd': (38884.8, 25711.9), 'bwd:ufc_fc1_wgrad_unfold': (61701.1, 6624.0), 'bwd:ufc_fc1_dgrad_unfold': (26078.5, 12611.2), 'bwd:wgrad_reduce': (14869.7, 1104.0)},
    'sampled_c512_h7': {'fwd:weight_prep': (6709.6, 1664.0), 'fwd:ufc_fc1_unfold': (7412.6, 6272.9), 'fwd:ufc_mid_fwd': (13052.4, 6322.7), 'fwd:ufc_fc2': (10617.0, 6272.0), 'bwd:ufc_fc2_wgrad': (12804.6, 8192.0), 'bwd:ufc_fc2_dgrad': (10616.9, 6272.0), 'bwd:ufc_mid_bwd': (19622.7, 12648.0), 'bwd:ufc_fc1_wgrad_unfold': (19711.7, 4608.0), 'bwd:ufc_fc1_dgrad_unfold': (13682.6, 6278.0), 'bwd:wgrad_reduce': (12855.8, 6656.0)},
    'chain_relu': {'fwd:chain_fwd': (50494.8, 56897.6), 'bwd:chain_bwd': (100764.7, 56030.4)},
    'chain_gate': {'fwd:chain_fwd': (50662.8, 57627.5), 'bwd:chain_bwd': (101068.1, 57927.8)},
    'chain_shift_residual': {'fwd:chain_fwd': (50649.2, 59868.6), 'bwd:chain_bwd': (100823.2, 57042.1)},
    'chain_box3': {'fwd:chain_fwd': (55416.3, 51561.4), 'bwd:chain_bwd': (55409.9, 51586.4)},
    'chain_softmax_c': {'fwd:chain_fwd': (100595.2, 55565.5), 'bwd:chain_bwd': (251269.7, 53517.8)},
    'fuzz': {'all:chain': (64858.9, 44338.0)},
}


def traffic_hash():
    import glob
    import hashlib

    # files of the source folder that hold no kernel and no launch logic of the workloads in the table (blocks composed
    # of several plans, templates and their solvers) are left out
    _NOT_MEASURED = {"block.hip", "plan_calls.hpp", "template.cpp", "symbolic.cpp", "symbolic.hpp"}
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2304_07741_amd", "csrc", "*"))):
        if os.path.basename(f) not in _NOT_MEASURED:
            h.update(open(f, "rb").read())
    return h.hexdigest()


_traffic_valid = None


def measured_traffic(workload, phase, kernel):
    global _traffic_valid
    t = TRAFFIC_KIB.get(workload, {}).get(f"{phase}:{kernel}")
    if t is None:
        return None
    if _traffic_valid is None:
        try:
            _traffic_valid = traffic_hash() == TRAFFIC_SHA256
        except OSError:
            _traffic_valid = False
    return (t[0] + t[1]) * 1024.0 if _traffic_valid else None


def make_case(name, batch=None):
    from paper_2304_07741_amd import workloads as wl

    kw = {} if batch is None else {"N": int(batch)}
    if name == "shift_residual":
        return wl.config2(**kw)
    if name.startswith("shift_residual_c"):  # shift_residual_cC_hH: the same DAG at another shape (C/4 channels per FC group)
        c, h = name[len("shift_residual_c"):].split("_h")
        return wl.config2(C=int(c), H=int(h), **kw)
    if name == "involution":
        return wl.config3(**kw)
    if name.startswith("sampled_c"):
        c, h = name[len("sampled_c"):].split("_h")
        return wl.config4(int(c), int(h), **kw)
    if name.startswith("chain_"):  # chain_<body>[_cC_hH]: an FC-free chain of memory-bound primitives
        import re

        body, c, h = name[len("chain_"):], 64, 56
        m = re.fullmatch(r"(.*)_c(\d+)_h(\d+)", body)
        if m:
            body, c, h = m.group(1), int(m.group(2)), int(m.group(3))
        if body not in wl.CHAIN_BODIES:
            raise SystemExit(f"unknown chain {body}: one of {sorted(wl.CHAIN_BODIES)}")
        return wl.chain(body, C=c, H=h, **kw)
    raise SystemExit(f"unknown workload {name}")


def infer_latency(args):
    """Forward-only latency of the inference plan at a small batch: eager calls and replays of one HIP graph
    that holds the forward launches (the library neither allocates nor synchronises, so it can be captured)."""
    import torch

    from paper_2304_07741_amd import binding as B
    from paper_2304_07741_amd import harness

    case = make_case(args.workload, args.infer)
    flags = (B.CANVAS_OPT_NO_FUSION if args.no_fusion else 0) | B.CANVAS_OPT_INFERENCE
    r = harness.DagRunner(case["blob"], case["shape"], case["dtype"], flags)
    r.load(case["x"], case["weights"])
    r.prepare()
    for _ in range(args.warmup):
        r.forward()
    torch.cuda.synchronize()

    def timed(fn):
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return 1e3 * (time.perf_counter() - t0) / args.steps

    eager_ms = timed(r.forward)
    y_eager = r.y.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        r.forward()
        with torch.cuda.graph(g, stream=side):
            r.forward()
    torch.cuda.synchronize()
    r.y.zero_()
    g.replay()
    torch.cuda.synchronize()
    same = bool(torch.equal(r.y, y_eager))
    graph_ms = timed(g.replay)
    B.canvas_dag_set_timing(r.handle, 1)
    nf = r.info.n_launches_fwd
    acc = [0.0] * nf
    for _ in range(20):
        r.forward()
        for k, ms in enumerate(B.canvas_dag_get_timing(r.handle, 0, nf)):
            acc[k] += ms / 20
    B.canvas_dag_set_timing(r.handle, 0)
    N = case["shape"][0]
    print(json.dumps({
        "metric": "micro-DAG forward latency, inference plan", "value": eager_ms, "unit": "ms", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": eager_ms, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": case["dtype"], "data": "synthetic",
        "config": {"workload": f"{case['name']} N={N} C={case['shape'][1]} H=W={case['shape'][2]} {case['dtype']} (seed {case['seed']})",
                   "fused": bool(r.info.fused), "launches_fwd": nf, "launches_prepare": r.info.n_launches_prepare},
        "eager_ms": eager_ms, "graph_ms": graph_ms, "graph_equals_eager": same, "kernel_sum_ms": sum(acc),
        "images_per_s_graph": N / (graph_ms * 1e-3),
        "kernels": [{"name": d["name"], "ms": round(acc[k], 5)} for k, d in enumerate(r.launches(0))]}))


def cpu_baseline(case, budget_s=12.0):
    """The oracle as it stands, timed on the host cores on the same workload (whole batch, repeated)."""
    import numpy as np

    from oracle import canvas_oracle
    from paper_2304_07741_amd import workloads as wl

    x = case["x"].astype(np.float64)
    ws = [w.astype(np.float64) for w in case["weights"]]
    ref = canvas_oracle.run(case["blob"], x, ws)
    dy = wl.make_dy(case, ref["y"].shape).astype(np.float64)
    times, threads = [], 1
    t_end = time.time() + budget_s
    while len(times) < 3 or (time.time() < t_end and len(times) < 15):
        t0 = time.perf_counter()
        r = canvas_oracle.run(case["blob"], x, ws, dy)
        times.append(time.perf_counter() - t0)
        threads = r["threads"]
    N = case["shape"][0]
    return {"value": N / statistics.median(times), "unit": "images/s", "cores": int(threads), "kind": "oracle",
            "sample": f"whole batch of {N} images, forward+backward, median of {len(times)} runs, "
                      f"gcc {' '.join(canvas_oracle.CFLAGS[:2])}, OpenMP over the batch index"}


def copy_reference(args):
    """A plain copy of one activation tensor of the workload, rotating over enough buffer pairs to stay cold."""
    import torch

    case = make_case(args.workload)
    n = 1
    for d in case["shape"]:
        n *= d
    esz = 2 if case["dtype"] == "bf16" else 4
    sets = max(2, min(16, int(2 * (512 << 20) / (2 * n * esz)) + 1))
    dt = torch.bfloat16 if esz == 2 else torch.float32
    src = [torch.randn(n, device="cuda").to(dt) for _ in range(sets)]
    dst = [torch.empty(n, device="cuda", dtype=dt) for _ in range(sets)]
    for i in range(args.warmup):
        dst[i % sets].copy_(src[i % sets])
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    for i, (a, b) in enumerate(ev):
        a.record()
        dst[i % sets].copy_(src[i % sets])
        b.record()
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(b) for a, b in ev)
    med = ms[len(ms) // 2]
    print(json.dumps({"metric": "plain device copy (torch copy kernel), bytes read + written per second", "value": 2 * n * esz / med / 1e6,
                      "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": med,
                      "higher_is_better": True, "dtype": case["dtype"], "data": "synthetic",
                      "config": {"workload": "copy of one activation tensor of " + args.workload, "bytes_in": n * esz, "bytes_out": n * esz,
                                 "buffer_pairs": sets, "ms_min": ms[0]}}))


def measure(case, flags, steps, warmup, rotate=True, kernel_steps=50):
    """W warm-up + K timed steps (forward + backward) of one workload, then the same steps with HIP events around every
    launch.  Returns ms per step, the per-launch list and the first runner's plan info."""
    import torch

    from paper_2304_07741_amd import binding as B
    from paper_2304_07741_amd import harness
    from paper_2304_07741_amd import workloads as wl

    first = harness.DagRunner(case["blob"], case["shape"], case["dtype"], flags)
    oshape = first.out_shape if first.out_shape[2] != 1 else (first.out_shape[0], first.out_shape[1], *first.out_shape[3:])
    dy = wl.make_dy(case, oshape)
    # rotate buffer sets: > 2x the last-level cache in total, at most 8 sets (rotate=False: operands stay in cache)
    per_set = sum(t.numel() * t.element_size() for t in (first.x, first.y, first.dy, first.dx)) + int(first.info.workspace_bytes)
    n_sets = max(2, min(8, -(-600_000_000 // per_set))) if rotate else 1
    runners = [first] + [harness.DagRunner(case["blob"], case["shape"], case["dtype"], flags) for _ in range(n_sets - 1)]
    for r in runners:
        r.load(case["x"], case["weights"], dy)
    torch.cuda.synchronize()

    def step(i):
        r = runners[i % n_sets]
        r.forward()
        r.backward()

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    ms_per_step = 1e3 * (time.perf_counter() - t0) / steps

    nf, nb = first.info.n_launches_fwd, first.info.n_launches_bwd
    for r in runners:
        B.canvas_dag_set_timing(r.handle, 1)
    acc = [[0.0] * nf, [0.0] * nb]
    psteps = max(1, min(steps, kernel_steps))
    for i in range(psteps):
        r = runners[i % n_sets]
        r.forward()
        r.backward()
        for b, n in ((0, nf), (1, nb)):
            for k, ms in enumerate(B.canvas_dag_get_timing(r.handle, b, n)):
                acc[b][k] += ms / psteps
    for r in runners:
        B.canvas_dag_set_timing(r.handle, 0)
    launches = []
    for b in (0, 1):
        for k, d in enumerate(first.launches(b)):
            launches.append({"phase": "bwd" if b else "fwd", "name": d["name"], "ms": acc[b][k], "bytes": d["bytes"], "flops": d["flops"]})
    info = {"fused": bool(first.info.fused), "chains": int(first.info.n_fused_chains), "chain_nodes": int(first.info.n_fused_nodes),
            "buffer_sets": n_sets, "launches_fwd": nf, "launches_bwd": nb, "workspace_bytes": int(first.info.workspace_bytes),
            "min_bytes": first.info.min_bytes_fwd + first.info.min_bytes_bwd}
    for r in runners:
        r.close()
    del runners, first
    torch.cuda.empty_cache()
    return ms_per_step, launches, info


def roofline_of(launches, workload, fused):
    """The slowest launch against the roof that binds it (its own algorithmic bytes / flops)."""
    dom = max(launches, key=lambda l: l["ms"])
    hbm_t = dom["bytes"] / (HBM_PEAK_GBS * 1e9)
    mfma_t = dom["flops"] / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    if mfma_t > hbm_t:
        ach = dom["flops"] / (dom["ms"] * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS,
                "traffic": None}
    else:
        ach = dom["bytes"] / (dom["ms"] * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "traffic": None}
    if fused:
        roof["traffic"] = measured_traffic(workload, dom["phase"], dom["name"])
    roof["kernel"] = f"{dom['name']} ({dom['phase']})"
    roof["kernel_ms"] = dom["ms"]
    roof["algorithmic_bytes"] = dom["bytes"]
    roof["algorithmic_flops"] = dom["flops"]
    return roof


def kernel_rows(launches):
    return [{"phase": l["phase"], "name": l["name"], "ms": round(l["ms"], 5), "GBps": round(l["bytes"] / max(l["ms"], 1e-9) / 1e6, 1),
             "TFLOPps": round(l["flops"] / max(l["ms"], 1e-9) / 1e9, 2)} for l in launches]


PER_CONFIG = ["involution", "sampled_c64_h56", "sampled_c128_h28", "sampled_c256_h14", "sampled_c512_h7"]


def fuzz_bench(args):
    """Config 5: the 200 random micro-DAGs (seeds 100-299), each timed for a few steps; geometric mean of images/s, how
    much of it runs in fused chains, and what the chain kernels reach against their algorithmic bytes."""
    import math

    from paper_2304_07741_amd import binding as B
    from paper_2304_07741_amd import workloads as wl

    lo, hi = (int(v) for v in args.seeds.split(":"))
    flags = B.CANVAS_OPT_NO_FUSION if args.no_fusion else 0
    logs, chain_ms, chain_bytes, all_ms, nf, nb, fully, with_chain = 0.0, 0.0, 0.0, 0.0, 0, 0, 0, 0
    slowest = None
    ratio_logs, faster = 0.0, 0  # --compare: every DAG also with one kernel per node, right after the fused run
    for seed in range(lo, hi):
        case = wl.config5(seed)
        ms, launches, info = measure(case, flags, args.steps, args.warmup, kernel_steps=min(args.steps, 10))
        if args.compare and not args.no_fusion:
            ms_nodes, _, _ = measure(case, B.CANVAS_OPT_NO_FUSION, args.steps, args.warmup, kernel_steps=1)
            ratio_logs += math.log(ms / ms_nodes)
            faster += 1 if ms < ms_nodes else 0
        logs += math.log(case["shape"][0] / (ms * 1e-3))
        for l in launches:
            all_ms += l["ms"]
            if l["name"].startswith("chain_"):
                chain_ms += l["ms"]
                chain_bytes += l["bytes"]
        nf += info["launches_fwd"]
        nb += info["launches_bwd"]
        with_chain += 1 if info["chains"] else 0
        fully += 1 if info["chains"] and not any(l["name"].startswith("node_") and "fc" not in l["name"] for l in launches) else 0
        if slowest is None or ms > slowest[1]:
            slowest = (seed, ms)
    n = hi - lo
    gm = math.exp(logs / n)
    frac = chain_bytes / max(chain_ms * 1e-3, 1e-12) / (HBM_PEAK_GBS * 1e9)
    out = {
        "metric": "micro-DAG fwd+bwd images/sec at ResNet layer shapes; % HBM / MFMA roofline",
        "value": gm, "unit": "images/s (geometric mean over the DAGs)", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 16.0 / gm * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"fuzz: random micro-DAGs, seeds {lo}-{hi - 1}, N=16 C=96 H=W=32 bf16", "dags": n, "with_fused_chains": with_chain,
                   "fully_fused": fully, "mean_launches_fwd": nf / n, "mean_launches_bwd": nb / n, "fusion": not args.no_fusion,
                   "slowest_seed": slowest[0], "slowest_ms": slowest[1]},
        "roofline": {"bound": "hbm", "achieved": frac * HBM_PEAK_GBS, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": frac,
                     # (bytes per DAG, like algorithmic_bytes; taken on the default seed range with fusion)
                     "traffic": measured_traffic("fuzz", "all", "chain") if (lo, hi) == (100, 300) and not args.no_fusion else None,
                     "kernel": "chain_fwd + chain_bwd, all DAGs (algorithmic bytes of every chain launch / summed kernel time)",
                     "kernel_ms": chain_ms / n, "algorithmic_bytes": chain_bytes / n},
        "chain_time_share": chain_ms / max(all_ms, 1e-12),
    }
    if args.compare and not args.no_fusion:
        out["against_one_kernel_per_node"] = {"geomean_step_time_ratio": math.exp(ratio_logs / n), "dags_faster": faster, "dags_slower": n - faster}
    print(json.dumps(out))


def block_bench(args):
    """A block with C_in != C_out composed from the shift + grouped FC + ReLU + residual template (include/canvas_block.h):
    block_<C_in>_<C_out> at N=64, H=W=56, bf16.  A step is forward + backward of the whole block; the roofline entry is the
    whole step against the bytes a block must move (x, dy read, y, dx written, once each), since the instances' launches
    are timed together."""
    import torch

    from paper_2304_07741_amd import harness
    from paper_2304_07741_amd import workloads as wl

    c_in, c_out = (int(v) for v in args.workload[len("block_"):].split("_"))
    c = min(c_in, c_out)
    n, h = 64, 56
    case = wl.block_case("block_shift_residual", wl.blob_shift_residual(c), (n, c_in, h, h), c_out, "bf16", 11,
                         [(4, c // 4, c // 4)], [1.0 / math.sqrt(c // 4)])
    act_bytes = 2.0 * n * h * h * (c_in + c_out)              # x and y (or dy and dx) once
    sets = max(2, int(2 * 256e6 / (2 * act_bytes)) + 1)      # rotate over more than twice the last-level cache
    runners = [harness.BlockRunner(case["blob"], case["shape"], c_out, "bf16") for _ in range(sets)]
    for r in runners:
        r.load(case["x"], case["weights"], case["dy"])
    from paper_2304_07741_amd import binding as B

    def step(r):
        B.canvas_block_forward(r.handle, r.x, r.w, r.y, r.ws)
        B.canvas_block_backward(r.handle, r.x, r.w, r.dy, r.dx, r.dw, r.ws)

    for i in range(args.warmup):
        step(runners[i % sets])
    torch.cuda.synchronize()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    for i in range(args.steps):
        step(runners[i % sets])
    t1.record()
    torch.cuda.synchronize()
    ms = t0.elapsed_time(t1) / args.steps
    info = runners[0].info
    alg = 2.0 * act_bytes
    ach = alg / (ms * 1e-3) / 1e9
    out = {"metric": "micro-DAG fwd+bwd images/sec at ResNet layer shapes; % HBM / MFMA roofline", "value": n / (ms * 1e-3), "unit": "images/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"block of {int(info.instances)} shift_residual templates, {'expand' if info.expand else 'reduce'}: "
                                  f"N={n} C_in={c_in} C_out={c_out} H=W={h} bf16 (seed 11)",
                      "instances": int(info.instances), "buffer_sets": sets, "workspace_bytes": int(info.workspace_bytes),
                      "launches_per_instance_fwd": int(info.plan.n_launches_fwd), "launches_per_instance_bwd": int(info.plan.n_launches_bwd)},
           "roofline": {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "traffic": None,
                        "kernel": "whole step (all instances, slice copies and sums)", "kernel_ms": ms, "algorithmic_bytes": alg}}
    if not args.no_cpu_baseline:
        import time

        from oracle import block_oracle

        k = 4  # images of the batch: a bounded sample
        x64 = case["x"][:k].astype("float64")
        t = time.perf_counter()
        block_oracle.run_block(case["blob"], x64, case["weights"], c_out, case["dy"][:k].astype("float64"))
        dt = time.perf_counter() - t
        out["cpu_baseline"] = {"value": k / dt, "unit": "images/s", "cores": os.cpu_count(), "kind": "oracle",
                               "sample": f"{k} images of the batch, forward+backward of every instance, one run"}
    for r in runners:
        r.close()
    print(json.dumps(out))


def fc_micro(args):
    """Grouped FC with its operands in cache: the contraction launches of config 4 at its four shapes, the same buffers
    every step (6-50 MB, far below the 256 MB last-level cache), each against the bf16 MFMA peak."""
    rows = []
    for name in PER_CONFIG[1:]:
        case = make_case(name)
        ms, launches, info = measure(case, 0, args.steps, args.warmup, rotate=False)
        for l in launches:
            if l["flops"] > 0:
                tf = l["flops"] / (l["ms"] * 1e-3) / 1e12
                rows.append({"workload": name, "phase": l["phase"], "kernel": l["name"], "ms": round(l["ms"], 5), "GFLOP": round(l["flops"] / 1e9, 3),
                             "TFLOPps": round(tf, 1), "frac_of_mfma_peak": round(tf / MFMA_BF16_PEAK_TFLOPS, 4)})
    best = max(rows, key=lambda r: r["TFLOPps"])
    print(json.dumps({"metric": "grouped-FC contraction kernels, operands in cache: TFLOP/s against the bf16 MFMA peak", "value": best["TFLOPps"],
                      "unit": "TFLOP/s (best kernel)", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": best["ms"],
                      "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": "FC launches of the sampled DAG at (C,H) in (64,56) (128,28) (256,14) (512,7), N=128, no buffer rotation"},
                      "roofline": {"bound": "mfma", "achieved": best["TFLOPps"], "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                   "frac": best["TFLOPps"] / MFMA_BF16_PEAK_TFLOPS, "traffic": None, "kernel": f"{best['kernel']} ({best['workload']})"},
                      "kernels": rows}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="shift_residual",
                    help="shift_residual (config 2, the headline), involution (config 3), sampled_cC_hH (config 4), fuzz (config 5)")
    ap.add_argument("--seeds", default="100:300", help="fuzz: range of seeds lo:hi")
    ap.add_argument("--compare", action="store_true", help="fuzz: time every DAG with one kernel per node as well and report the ratio")
    ap.add_argument("--no-fusion", action="store_true", help="per-node lowering (for comparison)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true", help="headline workload only: skip the per_config runs of configs 3 and 4")
    ap.add_argument("--infer", type=int, default=0, metavar="BATCH",
                    help="instead of the training step: forward-only latency of the inference plan at this batch size")
    ap.add_argument("--copy-ref", action="store_true",
                    help="instead of a micro-DAG: the rate of a plain device copy of one activation tensor of the workload "
                         "(torch's copy kernel, cold buffers), the reference that kernel times are compared with")
    ap.add_argument("--fc-micro", action="store_true", help="instead: the grouped-FC kernels of config 4 with their operands in cache")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)")
    if args.infer:
        return infer_latency(args)
    if args.copy_ref:
        return copy_reference(args)
    if args.fc_micro:
        return fc_micro(args)
    if args.workload.startswith("block_"):
        return block_bench(args)
    if args.workload == "fuzz":
        if args.steps == 200:
            args.steps, args.warmup = 10, 3
        return fuzz_bench(args)

    from paper_2304_07741_amd import binding as B

    case = make_case(args.workload)
    N = case["shape"][0]
    flags = B.CANVAS_OPT_NO_FUSION if args.no_fusion else 0
    ms_per_step, launches, info = measure(case, flags, args.steps, args.warmup)
    roof = roofline_of(launches, args.workload, not args.no_fusion)
    out = {
        "metric": "micro-DAG fwd+bwd images/sec at ResNet layer shapes; % HBM / MFMA roofline",
        "value": N / (ms_per_step * 1e-3), "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": case["dtype"], "data": "synthetic",
        "config": {"workload": f"{case['name']} N={case['shape'][0]} C={case['shape'][1]} H=W={case['shape'][2]} "
                               f"{case['dtype']} (seed {case['seed']})",
                   "fused": info["fused"], "fused_chains": info["chains"], "buffer_sets": info["buffer_sets"],
                   "launches_fwd": info["launches_fwd"], "launches_bwd": info["launches_bwd"], "workspace_bytes": info["workspace_bytes"]},
        "roofline": roof,
        "kernels": kernel_rows(launches),
        "min_bytes_fwd_bwd": info["min_bytes"],
        "whole_dag_hbm_frac": info["min_bytes"] / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9),
    }
    if args.workload == "shift_residual" and not args.no_per_config and not args.no_fusion:
        # the other configurations of the metric (ResNet-50 layer shapes and the dynamic-window DAG): fewer steps each
        per = []
        for name in PER_CONFIG:
            c = make_case(name)
            k = max(10, min(args.steps, 60))
            ms, ls, inf = measure(c, 0, k, max(3, min(args.warmup, 10)))
            r = roofline_of(ls, name, True)
            per.append({"workload": f"{c['name']} N={c['shape'][0]} C={c['shape'][1]} H=W={c['shape'][2]} {c['dtype']} (seed {c['seed']})",
                        "steps": k, "ms_per_step": ms, "images_per_s": c["shape"][0] / (ms * 1e-3), "launches_fwd": inf["launches_fwd"],
                        "launches_bwd": inf["launches_bwd"], "dominant_kernel": r["kernel"], "kernel_ms": r["kernel_ms"], "bound": r["bound"],
                        "achieved": r["achieved"], "unit": r["unit"], "frac": r["frac"], "traffic": r["traffic"],
                        "algorithmic_bytes": r["algorithmic_bytes"], "algorithmic_flops": r["algorithmic_flops"],
                        "whole_dag_hbm_frac": inf["min_bytes"] / (ms * 1e-3) / (HBM_PEAK_GBS * 1e9),
                        "fc_tflops": sum(l["flops"] for l in ls) / (ms * 1e-3) / 1e12})
        out["per_config"] = per
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(case)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
