"""Benchmark of the DeepPoly back-substitution hot path on one MI355X.

A step is one pass of the whole hot path (all layers' traversals, concretisations, margin rows and
verdicts) over one batch of synthetic boxes of the named workload.  The headline line is cfg5, the
largest configuration (9.9 TFLOP of back-substitution per step); the default run also measures every
other configuration the same way and reports them under "per_config" (cfg2: the three perturbation
sizes, 96 instances per step).  Inputs are resident in HBM before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0


def counter_traffic(workload):
    """L2-miss traffic of the dominant MFMA kernel per launch in bytes (fetch + write, calibrated on a plain copy of
    known size), as the committed rocprofv3 --pmc summary of this workload states it; None when there is none."""
    try:
        text = open(os.path.join(ROOT, "profiles", f"pmc_{workload}.txt")).read()
    except OSError:
        return None
    m = re.search(r"HBM traffic per launch.*total ([0-9.e+]+) bytes", text)
    return float(m.group(1)) if m else None


DESCR = {
    "cfg1": "cfg1: FC 784-100-100-100-10, B=1, eps=0.01",
    "cfg2": "cfg2: FC 784-6x500-10, B=32, eps in {0.005,0.01,0.02} (96 instances per step)",
    "cfg3": "cfg3: conv16 4x4s2 - conv32 4x4s2 - FC100 - FC10 on 3x32x32, B=32, eps=2/255",
    "cfg4": "cfg4: conv32 3x3 - conv32 4x4s2 - conv64 3x3 - conv64 4x4s2 - FC512 - FC512 - FC10 on 3x32x32, B=16, eps=1/255",
    "cfg5": "cfg5: FC 1024-9x1024-10, B=64, eps=0.005",
    "res_fc": "res_fc: residual FC 784-512-3x[512,512,+skip]-10, B=32, eps=0.001",
    "res_conv": "res_conv: residual conv16 3x3 - 2x[conv16 3x3, conv16 3x3, +skip] - conv32 4x4s2 - FC100 - FC10 on 1x28x28, B=16, eps=0.003",
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg5", choices=sorted(DESCR))
    ap.add_argument("--no-per-config", action="store_true", help="measure --workload only (profiler runs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=0, help="inputs per eps given to the CPU oracle (0 = default)")
    ap.add_argument("--variant", type=int, default=-1, help="contraction tile variant (tuning)")
    ap.add_argument("--certifier", default="deeppoly", choices=["deeppoly", "reusecert"],
                    help="reusecert: the NEXT-row certifier (fully-connected workloads only); default deeppoly is the headline")
    ap.add_argument("--max-depth", type=int, default=-1,
                    help="p >= 0: DeepPoly_p (at most p traverse iterations, then concretise against stored bounds); 0 = IBP")
    ap.add_argument("--final-depth", type=int, default=-2,
                    help="traversal limit of the last layer and margins (-2: same as --max-depth); --max-depth 0 --final-depth -1 = CROWN-IBP")
    ap.add_argument("--host-inputs", action="store_true", help="pass host arrays (adds the PCIe upload of the boxes to every step)")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE", help="dpc_tuning_set(KEY, VALUE) before the run")
    ap.add_argument("--fuse", type=int, default=1)
    ap.add_argument("--use-graph", type=int, default=-1, help="dpc_options.use_graph (-1: the library default)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run one plain 256 MiB device-to-device copy first (known size, to scale rocprofv3 byte counters)")
    return ap.parse_args()


# inputs per eps setting handed to the float64 oracle for the CPU baseline (bounded: a few seconds to ~15 s each)
CPU_SAMPLE = {"cfg1": 1, "cfg2": 32, "cfg3": 32, "cfg4": 2, "cfg5": 16, "res_fc": 16, "res_conv": 2}


def measure(workload, args, steps, warmup, cpu_baseline):
    """Times `steps` steps of one workload; returns the record (the headline line's fields for that workload)."""
    import numpy as np
    import torch
    from paper_2507_20055_amd import binding, workloads as wl

    n_eps = len(wl.CONFIGS[workload]["eps"])
    loads = [wl.make_workload(workload, eps_index=i) for i in range(n_eps)]
    net = binding.Network(loads[0].net, device=0)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        dev = [(torch.from_numpy(w.lo).cuda(), torch.from_numpy(w.hi).cuda(), torch.from_numpy(w.label).cuda()) for w in loads]
    stream.synchronize()
    if args.host_inputs:
        dev = [(w.lo, w.hi, w.label) for w in loads]
    B = loads[0].lo.shape[0]
    results = [None] * n_eps

    def step(profile):
        for i, (lo, hi, lab) in enumerate(dev):
            results[i] = net.certify(lo, hi, lab, stream=stream.cuda_stream, profile=profile, fuse=args.fuse, reuse=results[i], **({} if args.use_graph < 0 else {"use_graph": args.use_graph}),
                                     certifier=args.certifier, max_backsub_depth=args.max_depth,
                                     final_backsub_depth=args.final_depth)

    for _ in range(warmup):
        step(0)
    torch.cuda.synchronize()
    # timed region: K steps as a caller would run them
    t0 = time.perf_counter()
    for _ in range(steps):
        step(0)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # the same K steps again with HIP events recorded on the launch stream at every change of kernel class
    # (per-class durations for the roofline figures; the events themselves cost a few percent)
    prof_tot = None
    t1 = time.perf_counter()
    for _ in range(steps):
        step(1)
        for r in results:
            p = r.profile()
            prof_tot = p if prof_tot is None else {k: prof_tot[k] + p[k] for k in p}
    torch.cuda.synchronize()
    dt_events = time.perf_counter() - t1

    inputs_per_step = B * n_eps
    verified = int(sum(int(r.verdict()[0].sum()) for r in results))
    min_abs_margin = float(min(float(np.abs(r.verdict()[1]).min()) for r in results))
    last = len(loads[0].net.layers)
    # mean width u - l of the output layer's bounds over the batch (every eps setting): shows at a glance whether the
    # perturbation is one the relaxation can still say something about, or the bounds have blown up
    widths = [float(np.mean(np.subtract(*r.concrete(last)[::-1]))) for r in results]

    P = prof_tot
    # dominant MFMA kernel: the LDS-resident traversal kernel where it runs, else the per-layer contraction
    dom = "chain" if P["chain_ms"] > P["contract_ms"] else "contract"
    dom_name = {"chain": "chain_kernel (whole traversal of a layer's rows: fp32 MFMA C*W per layer crossed, rows resident in LDS)",
                "contract": "contract / conv-transpose kernels (fp32 MFMA C*W of one traversal step)"}[dom]
    dom_ms, dom_flop, dom_launches = P[dom + "_ms"], P[dom + "_flop"], P[dom + "_launches"]
    dom_tflops = dom_flop / (dom_ms * 1e-3) / 1e12 if dom_ms > 0 else 0.0
    mfma_ms = P["chain_ms"] + P["contract_ms"]
    mfma_tflops = (P["chain_flop"] + P["contract_flop"]) / (mfma_ms * 1e-3) / 1e12 if mfma_ms > 0 else 0.0
    default_run = not args.tune and args.variant < 0 and args.fuse == 1 and args.certifier == "deeppoly" and args.max_depth < 0 and args.final_depth in (-2, -1)

    def hbm_pass(key):
        # launches of a few rows (the output / margin rows of the fully-connected workloads) finish out of L2 and are
        # launch-bound: time and launch count only; a bandwidth figure is given from 64 MB of rows per launch up
        ms, launches, nbytes = P[key + "_ms"], P[key + "_launches"], P[key + "_bytes"]
        rec = {"launches": launches, "ms_per_step": ms / steps}
        if launches and ms > 0 and nbytes / launches >= 64e6:
            gbs = nbytes / (ms * 1e-3) / 1e9
            rec.update({"achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS})
        return rec

    split_terms = dict(kv.partition("=")[::2] for kv in args.tune).get("contract_split", "0")

    mfma_peak = {"2": 2500.0 / 3.0, "3": 2500.0 / 6.0}.get(split_terms, PEAK_FP32_MFMA_TFLOPS)

    out = {
        "metric": "certified inputs/sec",
        "value": inputs_per_step * steps / dt,
        "unit": "inputs/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": dt / steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": {"0": "f32", "2": "bf16x3 (operands split into two bf16 terms, fp32 accumulation)",
                  "3": "bf16x6 (operands split into three bf16 terms, fp32 accumulation)"}[dict(kv.partition("=")[::2] for kv in args.tune).get("contract_split", "0")],
        "data": "synthetic",
        "config": {"workload": DESCR[workload], "inputs_per_step": inputs_per_step,
                   "verified": verified, "min_abs_margin": min_abs_margin, "mean_output_bound_width": sum(widths) / len(widths),
                   "fuse": args.fuse,
                   "inputs": "host" if args.host_inputs else "resident in HBM", "certifier": args.certifier, "max_backsub_depth": args.max_depth, "final_backsub_depth": args.final_depth},
        "roofline": {
            "kernel": dom_name,
            # the split-precision experiment runs 3 (6) bf16 MFMA products per fp32-equivalent multiply-add: its peak is the
            # dense bf16 figure divided by that count; everything else is priced against the fp32 MFMA peak
            "bound": "mfma", "achieved": dom_tflops, "peak": mfma_peak, "unit": "TFLOP/s",
            "frac": dom_tflops / mfma_peak,
            "launches": dom_launches, "avg_launch_ms": dom_ms / max(dom_launches, 1),
            "flop_per_launch": dom_flop / max(dom_launches, 1),
            "traffic": counter_traffic(workload) if default_run else None,
            "all_mfma_kernels": {"achieved": mfma_tflops, "frac": mfma_tflops / mfma_peak,
                                 "flop_per_step": (P["chain_flop"] + P["contract_flop"]) / steps,
                                 "ms_per_step": mfma_ms / steps},
        },
        # the row passes left outside the MFMA kernels' epilogues in this run (the kernels themselves are measured
        # standalone below)
        "hbm_passes_in_run": {"relax_step": hbm_pass("relax"), "concretise": hbm_pass("concretise")},
        "time_split_ms_per_step": {k: P[k] / steps for k in ("chain_ms", "contract_ms", "relax_ms", "concretise_ms", "other_ms", "total_ms")},
        "value_with_kernel_events": inputs_per_step * steps / dt_events,
    }

    # The two HBM-bound passes as standalone kernels at this workload's dominant shape (both sides of the widest
    # hidden layer's rows over the widest layer below), timed with events on the launch stream.
    sizes = net.sizes
    hidden = [n for n, k in zip(sizes[1:], net.kinds) if k == "affine"]
    if len(hidden) >= 2:
        R, n = max(hidden[:-1]), max(sizes[:-1][:len(sizes) - 2] or [sizes[0]])
        n = min(n, 4096)
        ld = (n + 31) // 32 * 32
        M = 2 * B * R
        with torch.cuda.stream(stream):
            C = torch.randn(M, ld, device="cuda")
            cst = torch.zeros(M, device="cuda", dtype=torch.float64)
            lam, mu, nu = (torch.rand(B, n, device="cuda") for _ in range(3))
            bias = torch.randn(n, device="cuda")
            lo_ = torch.rand(B, n, device="cuda")
            hi_ = lo_ + 0.1
            ol, ou = torch.empty(B, R, device="cuda"), torch.empty(B, R, device="cuda")

            def timed(f, reps=20):
                for _ in range(3):
                    f()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for _ in range(reps):
                    f()
                e1.record(stream)
                e1.synchronize()
                return e0.elapsed_time(e1) / reps * 1e-3

            t_relax = timed(lambda: binding.dpc_op_relax_step(C, cst, 2, B, R, n, lam, mu, nu, bias, stream=stream.cuda_stream))
            t_conc = timed(lambda: binding.dpc_op_concretise(C, cst, 2, B, R, n, lo_, hi_, ol, ou, stream=stream.cuda_stream))
            # what a plain device-to-device copy of the same rows reaches at this size (the runtime's copy kernel; the same
            # bytes as the ReLU step: every row read once and written once): launch ramp and tail weigh the same on it
            C2 = torch.empty_like(C)
            t_copy = timed(lambda: C2.copy_(C))
            del C2
        out["hbm_passes_standalone"] = {
            "shape": {"rows": M, "columns": n},
            "relax_step": {"achieved": M * n * 8 / t_relax / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                           "frac": M * n * 8 / t_relax / 1e9 / PEAK_HBM_GBS, "us_per_launch": t_relax * 1e6},
            "concretise": {"achieved": M * n * 4 / t_conc / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                           "frac": M * n * 4 / t_conc / 1e9 / PEAK_HBM_GBS, "us_per_launch": t_conc * 1e6},
            "plain_copy_same_rows": {"achieved": M * ld * 8 / t_copy / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                     "frac": M * ld * 8 / t_copy / 1e9 / PEAK_HBM_GBS, "us_per_launch": t_copy * 1e6},
        }
        del C, cst

    if cpu_baseline:
        import oracle
        cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)))
        ns = min(B, args.cpu_sample or CPU_SAMPLE[workload])
        tc = time.perf_counter()
        for w in loads:
            oracle.run(w.net, w.lo[:ns], w.hi[:ns], label=w.label[:ns], threads=cores, certifier=args.certifier,
                       max_depth=args.max_depth, max_depth_last=None if args.final_depth == -2 else args.final_depth)
        tcpu = time.perf_counter() - tc
        out["cpu_baseline"] = {"value": ns * n_eps / tcpu, "unit": "inputs/s", "cores": cores, "kind": "oracle",
                               "sample": f"first {ns} of {B} inputs of each of the {n_eps} eps settings, float64 oracle, {tcpu:.1f} s"}
    results.clear()
    net.close()
    return out


def verdict_check():
    """Both verdicts in one line: the cfg2 network at eps = 0.001 -- a perturbation small enough that most inputs are
    certified (NOT one of the named settings, whose bounds are too wide to certify anything on untrained networks) --
    through the GPU path and through the oracle."""
    import numpy as np
    import oracle
    from paper_2507_20055_amd import binding, workloads as wl
    w = wl.make_workload("cfg2")
    eps = 0.001
    lo = np.clip(w.x - eps, 0.0, 1.0).astype(np.float32)
    hi = np.clip(w.x + eps, 0.0, 1.0).astype(np.float32)
    net = binding.Network(w.net, device=0)
    v, m = net.certify(lo, hi, w.label).verdict()
    net.close()
    o = oracle.run(w.net, lo, hi, label=w.label)
    return {"workload": "cfg2 network, B=32, eps=0.001 (not a named setting)", "inputs": int(v.size), "verified": int(v.sum()),
            "oracle_verified": int(o.verdict.sum()), "verdicts_identical": bool(np.array_equal(v, o.verdict)),
            "min_margin": float(m.min()), "max_margin": float(m.max())}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2507_20055_amd import binding

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.variant >= 0:
        binding.dpc_tuning_set("contract_variant", args.variant)
    for kv in args.tune:
        key, _, val = kv.partition("=")
        binding.dpc_tuning_set(key, int(val))

    if args.calibrate_copy:
        src = torch.empty(64 * 1024 * 1024, device="cuda", dtype=torch.float32).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    out = measure(args.workload, args, args.steps, args.warmup, not args.no_cpu_baseline)
    if not args.no_per_config and args.workload == "cfg5":
        # every other configuration, measured the same way in this same run (each its own timed region of K steps)
        per = []
        for name in ("cfg1", "cfg2", "cfg3", "cfg4", "res_fc", "res_conv"):
            if args.certifier == "reusecert" and name in ("res_fc", "res_conv"):
                continue
            r = measure(name, args, args.steps, args.warmup, not args.no_cpu_baseline)
            rec = {"workload": r["config"]["workload"], "value": r["value"], "unit": r["unit"], "ms_per_step": r["ms_per_step"],
                   "inputs_per_step": r["config"]["inputs_per_step"], "verified": r["config"]["verified"],
                   "mean_output_bound_width": r["config"]["mean_output_bound_width"],
                   "roofline": {k: r["roofline"][k] for k in ("kernel", "bound", "achieved", "peak", "unit", "frac", "launches", "avg_launch_ms", "traffic")},
                   "all_mfma_kernels_frac": r["roofline"]["all_mfma_kernels"]["frac"],
                   "time_split_ms_per_step": r["time_split_ms_per_step"]}
            if "hbm_passes_standalone" in r:
                h = r["hbm_passes_standalone"]
                rec["hbm_passes_standalone"] = {"shape": h["shape"], "relax_step_frac": h["relax_step"]["frac"], "concretise_frac": h["concretise"]["frac"]}
            if "cpu_baseline" in r:
                rec["cpu_baseline"] = r["cpu_baseline"]
            per.append(rec)
        out["per_config"] = per
        if not args.no_cpu_baseline and args.certifier == "deeppoly" and args.max_depth < 0:
            out["verdict_check"] = verdict_check()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
