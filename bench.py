"""Benchmark: forward+backward images/s of a micro-DAG kernel on one MI355X, with the roofline fraction
of its dominant kernel and the CPU oracle timed beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload shift_residual|involution|sampled_cC_hH]
    python bench.py --infer BATCH [--workload ...]     (forward-only latency of the inference plan, not the headline)

One step = one forward + one backward of the whole micro-DAG over one batch resident in HBM.  Buffer
sets are rotated so that consecutive steps do not find their operands in the 256 MB last-level cache.
Prints one JSON line.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0


# HBM bytes per launch from two `rocprofv3 --pmc` runs of this file (FETCH_SIZE, then WRITE_SIZE, KiB per
# dispatch; a plain 25 088 KiB copy reads FETCH_SIZE 12 554 -> factor 1.998, WRITE_SIZE 25 088 -> factor 1.0).
# Valid only for the kernel sources they were taken on (hash below), otherwise `traffic` is null.
TRAFFIC_SOURCES = ["paper_2304_07741_amd/csrc/sgfc_kernels.hip", "paper_2304_07741_amd/csrc/tile_util.hpp",
                   "paper_2304_07741_amd/csrc/lower_sgfc.cpp"]
TRAFFIC_SHA256 = "85f5cd49ad9d645defc73f2211fa19ebaec35cf5cf1d1246f1b1c66b132d7640"
TRAFFIC_KIB = {("shift_residual", "sgfc_bwd"): (26403.5 * 1.998, 25900.3), ("shift_residual", "sgfc_fwd"): (14405.3 * 1.998, 25089.0)}


def measured_traffic(workload, kernel):
    import hashlib

    h = hashlib.sha256()
    try:
        for f in TRAFFIC_SOURCES:
            h.update(open(os.path.join(ROOT, f), "rb").read())
    except OSError:
        return None
    if h.hexdigest() != TRAFFIC_SHA256 or (workload, kernel) not in TRAFFIC_KIB:
        return None
    fetch, write = TRAFFIC_KIB[(workload, kernel)]
    return (fetch + write) * 1024.0


def make_case(name, batch=None):
    from paper_2304_07741_amd import workloads as wl

    kw = {} if batch is None else {"N": int(batch)}
    if name == "shift_residual":
        return wl.config2(**kw)
    if name == "involution":
        return wl.config3(**kw)
    if name.startswith("sampled_c"):
        c, h = name[len("sampled_c"):].split("_h")
        return wl.config4(int(c), int(h), **kw)
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="shift_residual")
    ap.add_argument("--no-fusion", action="store_true", help="per-node lowering (for comparison)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--infer", type=int, default=0, metavar="BATCH",
                    help="instead of the training step: forward-only latency of the inference plan at this batch size")
    ap.add_argument("--copy-ref", action="store_true",
                    help="instead of a micro-DAG: the rate of a plain device copy of one activation tensor of the workload "
                         "(torch's copy kernel, cold buffers), the reference that kernel times are compared with")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)")
    if args.infer:
        return infer_latency(args)
    if args.copy_ref:
        return copy_reference(args)

    import torch

    from paper_2304_07741_amd import binding as B
    from paper_2304_07741_amd import harness
    from paper_2304_07741_amd import workloads as wl

    case = make_case(args.workload)
    N = case["shape"][0]
    flags = B.CANVAS_OPT_NO_FUSION if args.no_fusion else 0
    first = harness.DagRunner(case["blob"], case["shape"], case["dtype"], flags)
    oshape = first.out_shape if first.out_shape[2] != 1 else (first.out_shape[0], first.out_shape[1], *first.out_shape[3:])
    dy = wl.make_dy(case, oshape)
    # rotate buffer sets: > 2x the last-level cache in total, at most 8 sets
    per_set = sum(t.numel() * t.element_size() for t in (first.x, first.y, first.dy, first.dx)) + int(first.info.workspace_bytes)
    n_sets = max(2, min(8, -(-600_000_000 // per_set)))
    runners = [first] + [harness.DagRunner(case["blob"], case["shape"], case["dtype"], flags) for _ in range(n_sets - 1)]
    for r in runners:
        r.load(case["x"], case["weights"], dy)
    torch.cuda.synchronize()

    def step(i):
        r = runners[i % n_sets]
        r.forward()
        r.backward()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps

    # per-kernel durations: the same steps again with HIP events around every launch
    nf, nb = first.info.n_launches_fwd, first.info.n_launches_bwd
    for r in runners:
        B.canvas_dag_set_timing(r.handle, 1)
    acc = [[0.0] * nf, [0.0] * nb]
    psteps = min(args.steps, 50)
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
            launches.append({"phase": "bwd" if b else "fwd", "name": d["name"], "ms": acc[b][k], "bytes": d["bytes"],
                             "flops": d["flops"]})
    dom = max(launches, key=lambda l: l["ms"])
    hbm_t = dom["bytes"] / (HBM_PEAK_GBS * 1e9)
    mfma_t = dom["flops"] / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    if mfma_t > hbm_t:
        ach = dom["flops"] / (dom["ms"] * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": None}
    else:
        ach = dom["bytes"] / (dom["ms"] * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                "traffic": None}
    if roof["bound"] == "hbm" and not args.no_fusion:
        roof["traffic"] = measured_traffic(args.workload, dom["name"])
    roof["kernel"] = f"{dom['name']} ({dom['phase']})"
    roof["kernel_ms"] = dom["ms"]
    roof["algorithmic_bytes"] = dom["bytes"]

    out = {
        "metric": "micro-DAG fwd+bwd images/sec at ResNet layer shapes; % HBM / MFMA roofline",
        "value": N / (ms_per_step * 1e-3), "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": case["dtype"], "data": "synthetic",
        "config": {"workload": f"{case['name']} N={case['shape'][0]} C={case['shape'][1]} H=W={case['shape'][2]} "
                               f"{case['dtype']} (seed {case['seed']})",
                   "fused": bool(first.info.fused), "buffer_sets": n_sets,
                   "launches_fwd": nf, "launches_bwd": nb, "workspace_bytes": int(first.info.workspace_bytes)},
        "roofline": roof,
        "kernels": [{"phase": l["phase"], "name": l["name"], "ms": round(l["ms"], 5),
                     "GBps": round(l["bytes"] / max(l["ms"], 1e-9) / 1e6, 1),
                     "TFLOPps": round(l["flops"] / max(l["ms"], 1e-9) / 1e9, 2)} for l in launches],
        "min_bytes_fwd_bwd": first.info.min_bytes_fwd + first.info.min_bytes_bwd,
        "whole_dag_hbm_frac": (first.info.min_bytes_fwd + first.info.min_bytes_bwd) / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9),
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(case)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
