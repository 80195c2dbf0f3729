"""Benchmark of the DeepPoly back-substitution hot path on one MI355X.

A step is one pass of the whole hot path (all layers' traversals, concretisations, margin rows and
verdicts) over one batch of synthetic boxes of the named workload; for cfg2 that is the three
perturbation sizes, 96 instances.  Inputs are resident in HBM before the timed region.  Prints ONE
JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0

# L2-miss traffic of the dominant MFMA kernel per launch, bytes (fetch + write), from the two rocprofv3 --pmc
# runs summarised in profiles/pmc_<workload>.txt (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0 after calibration on a
# plain 256 MiB copy); mean over the launches of one step.  Only valid for the default tuning.
TRAFFIC = {"cfg2": 7.352e7, "cfg3": 1.540e8, "cfg4": 1.985e9, "cfg5": 2.561e9, "res_fc": 1.449e8, "res_conv": 1.136e9}

DESCR = {
    "cfg1": "cfg1: FC 784-100-100-100-10, B=1, eps=0.01",
    "cfg2": "cfg2: FC 784-6x500-10, B=32, eps in {0.005,0.01,0.02} (96 instances per step)",
    "cfg3": "cfg3: conv16 4x4s2 - conv32 4x4s2 - FC100 - FC10 on 3x32x32, B=32, eps=2/255",
    "cfg4": "cfg4: conv32 3x3 - conv32 4x4s2 - conv64 3x3 - conv64 4x4s2 - FC512 - FC512 - FC10 on 3x32x32, B=16, eps=1/255",
    "cfg5": "cfg5: FC 1024-9x1024-10, B=64, eps=0.005",
    "res_fc": "res_fc: residual FC 784-512-3x[512,512,+skip]-10, B=32, eps=0.001",
    "res_conv": "res_conv: residual conv16 3x3 - 2x[conv16 3x3, conv16 3x3, +skip] - conv32 4x4s2 - FC100 - FC10 on 1x28x28, B=16, eps=0.003",
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg2", choices=sorted(DESCR))
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
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2507_20055_amd import binding, workloads as wl

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

    n_eps = len(wl.CONFIGS[args.workload]["eps"])
    loads = [wl.make_workload(args.workload, eps_index=i) for i in range(n_eps)]
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

    for _ in range(args.warmup):
        step(0)
    torch.cuda.synchronize()
    # timed region: K steps as a caller would run them
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(0)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # the same K steps again with HIP events recorded on the launch stream at every change of kernel class
    # (per-class durations for the roofline figures; the events themselves cost a few percent)
    prof_tot = None
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step(1)
        for r in results:
            p = r.profile()
            prof_tot = p if prof_tot is None else {k: prof_tot[k] + p[k] for k in p}
    torch.cuda.synchronize()
    dt_events = time.perf_counter() - t1

    inputs_per_step = B * n_eps
    verified = int(sum(int(r.verdict()[0].sum()) for r in results))
    min_abs_margin = float(min(float(np.abs(r.verdict()[1]).min()) for r in results))

    P = prof_tot
    # dominant MFMA kernel: the LDS-resident traversal kernel where it runs, else the per-layer contraction
    dom = "chain" if P["chain_ms"] > P["contract_ms"] else "contract"
    dom_name = {"chain": "chain_kernel (whole traversal of a layer's rows: fp32 MFMA C*W per layer crossed, rows resident in LDS)",
                "contract": "contract / conv-transpose kernels (fp32 MFMA C*W of one traversal step)"}[dom]
    dom_ms, dom_flop, dom_launches = P[dom + "_ms"], P[dom + "_flop"], P[dom + "_launches"]
    dom_tflops = dom_flop / (dom_ms * 1e-3) / 1e12 if dom_ms > 0 else 0.0
    mfma_ms = P["chain_ms"] + P["contract_ms"]
    mfma_tflops = (P["chain_flop"] + P["contract_flop"]) / (mfma_ms * 1e-3) / 1e12 if mfma_ms > 0 else 0.0
    relax_gbs = P["relax_bytes"] / (P["relax_ms"] * 1e-3) / 1e9 if P["relax_ms"] > 0 else 0.0
    conc_gbs = P["concretise_bytes"] / (P["concretise_ms"] * 1e-3) / 1e9 if P["concretise_ms"] > 0 else 0.0

    out = {
        "metric": "certified inputs/sec",
        "value": inputs_per_step * args.steps / dt,
        "unit": "inputs/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": {"0": "f32", "2": "bf16x3 (operands split into two bf16 terms, fp32 accumulation)",
                  "3": "bf16x6 (operands split into three bf16 terms, fp32 accumulation)"}[dict(kv.partition("=")[::2] for kv in args.tune).get("contract_split", "0")],
        "data": "synthetic",
        "config": {"workload": DESCR[args.workload], "inputs_per_step": inputs_per_step,
                   "verified": verified, "min_abs_margin": min_abs_margin, "fuse": args.fuse,
                   "inputs": "host" if args.host_inputs else "resident in HBM", "certifier": args.certifier, "max_backsub_depth": args.max_depth, "final_backsub_depth": args.final_depth},
        "roofline": {
            "kernel": dom_name,
            "bound": "mfma", "achieved": dom_tflops, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
            "frac": dom_tflops / PEAK_FP32_MFMA_TFLOPS,
            "launches": dom_launches, "avg_launch_ms": dom_ms / max(dom_launches, 1),
            "flop_per_launch": dom_flop / max(dom_launches, 1),
            "traffic": TRAFFIC.get(args.workload) if not args.tune and args.variant < 0 and args.fuse == 1 and args.certifier == "deeppoly" and args.max_depth < 0 and args.final_depth in (-2, -1) else None,
            "all_mfma_kernels": {"achieved": mfma_tflops, "frac": mfma_tflops / PEAK_FP32_MFMA_TFLOPS,
                                 "flop_per_step": (P["chain_flop"] + P["contract_flop"]) / args.steps,
                                 "ms_per_step": mfma_ms / args.steps},
        },
        # the row passes left outside the MFMA kernels' epilogues in this run (on the fully-connected workloads
        # only the few margin / output rows: launch-bound; the kernels themselves are measured below)
        "hbm_passes_in_run": {
            "relax_step": {"achieved": relax_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": relax_gbs / PEAK_HBM_GBS,
                           "launches": P["relax_launches"], "ms_per_step": P["relax_ms"] / args.steps},
            "concretise": {"achieved": conc_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": conc_gbs / PEAK_HBM_GBS,
                           "launches": P["concretise_launches"], "ms_per_step": P["concretise_ms"] / args.steps},
        },
        "time_split_ms_per_step": {k: P[k] / args.steps for k in ("chain_ms", "contract_ms", "relax_ms", "concretise_ms", "other_ms", "total_ms")},
        "value_with_kernel_events": inputs_per_step * args.steps / dt_events,
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
        out["hbm_passes_standalone"] = {
            "shape": {"rows": M, "columns": n},
            "relax_step": {"achieved": M * n * 8 / t_relax / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                           "frac": M * n * 8 / t_relax / 1e9 / PEAK_HBM_GBS, "us_per_launch": t_relax * 1e6},
            "concretise": {"achieved": M * n * 4 / t_conc / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                           "frac": M * n * 4 / t_conc / 1e9 / PEAK_HBM_GBS, "us_per_launch": t_conc * 1e6},
        }
        del C, cst

    if not args.no_cpu_baseline:
        import oracle
        cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)))
        default_sample = {"cfg1": 1, "cfg2": 32, "cfg3": 32, "cfg4": 2, "cfg5": 16, "res_fc": 16, "res_conv": 2}[args.workload]
        ns = min(B, args.cpu_sample or default_sample)
        tc = time.perf_counter()
        for w in loads:
            oracle.run(w.net, w.lo[:ns], w.hi[:ns], label=w.label[:ns], threads=cores, certifier=args.certifier,
                       max_depth=args.max_depth, max_depth_last=None if args.final_depth == -2 else args.final_depth)
        tcpu = time.perf_counter() - tc
        out["cpu_baseline"] = {"value": ns * n_eps / tcpu, "unit": "inputs/s", "cores": cores, "kind": "oracle",
                               "sample": f"first {ns} of {B} inputs of each of the {n_eps} eps settings, float64 oracle, {tcpu:.1f} s"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
