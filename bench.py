#!/usr/bin/env python3
"""Benchmark of the unified/pruned-weight GEMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4|cfg5] [--report]

Headline workload (config.workload = "cfg4_decode_projections"): the transformer projection GEMMs of
the decode regime -- K = N = 4096, blocks of 16 along K, 70 % unified / 25 % pruned / 5 % dense, bf16,
M in {1, 8, 16}.  One such matrix is ~4.9 MB compressed, far below launch latency and below the cache
sizes, so a step streams G = 128 distinct encoded matrices (631 MB, more than the 256 MB of last-level
cache) through ONE muw_gemm_grouped launch per M: a step is three launches (M = 1, 8, 16).  All
inputs are resident in HBM before the timed region.  `value` is compressed-weight bytes per second.

The line printed on stdout is one JSON object; `roofline` describes the streaming kernel (algorithmic
bytes = compressed weights + activations + outputs per launch, against the 8 TB/s HBM peak) and
`cpu_baseline` times the CPU oracle on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 MFMA rate


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg4", choices=["cfg4", "cfg5"])
    ap.add_argument("--groups", type=int, default=128, help="distinct encoded matrices per launch (cfg4)")
    ap.add_argument("--distinct", type=int, default=4, help="matrices generated from distinct seeds (cfg4)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--report", action="store_true", help="also time the other configs (stderr + gpurun_out/report.json)")
    return ap.parse_args()


def traffic_from_profiles(kernel_key):
    """HBM bytes per launch measured with rocprofv3 --pmc (see profiles/), if recorded."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(path):
        return None
    try:
        return json.load(open(path)).get(kernel_key)
    except Exception:
        return None


def time_steps(torch, fn, steps, warmup):
    """Returns (wall ms per step, HIP-event ms per step).  Events are recorded on torch's current
    stream, which is the stream every launch of fn goes to."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    return wall, e0.elapsed_time(e1) / steps


def bench_cfg4(args, torch, muw, synth, to_device):
    G, ndist = args.groups, max(1, min(args.distinct, args.groups))
    case = synth.config4(16)
    t0 = time.time()
    base, host_W = [], []
    for i in range(ndist):
        W = synth.normal_tensor(case.seed + i, (case.N, case.K), case.w_std, "bf16", stream=1)
        base.append(muw.muw_encode(to_device(W), case.B, case.r_unify, case.r_prune))
        if i < 2:
            host_W.append(W)
    # G distinct device allocations (copies of the ndist encoded matrices): what matters to the
    # kernel is that every launch streams G separate blobs from HBM
    layers = [muw.EncodedLayer(base[g % ndist].desc, base[g % ndist].blob.clone()) for g in range(G)]
    groups, host_X = {}, {}
    for M in (1, 8, 16):
        Xs = []
        for g in range(G):
            X = synth.normal_tensor(case.seed + 100 + g, (M, case.K), 1.0, "bf16", stream=M)
            Xs.append(to_device(X))
            if g < 2:
                host_X[(M, g)] = X
        groups[M] = muw.GemmGroup(layers, Xs)
    log(f"[bench] cfg4 inputs: {G} blobs ({ndist} distinct), built in {time.time() - t0:.1f} s")

    def step():
        for M in (1, 8, 16):
            muw.muw_gemm_grouped(groups[M])

    wall_ms, ev_ms = time_steps(torch, step, args.steps, args.warmup)
    comp = sum(l.compressed_bytes for l in layers)
    per_M = {}
    for M in (1, 8, 16):
        _, ms = time_steps(torch, lambda: muw.muw_gemm_grouped(groups[M]), args.steps, 1)
        algo = comp + G * (M * case.K * 2 + M * case.N * 4)
        flops_surv = 2.0 * M * case.B * sum(l.NB - l.desc.n_pruned for l in layers)
        per_M[str(M)] = {"ms_per_launch": ms, "compressed_GBps": comp / ms / 1e6,
                         "algorithmic_GBps": algo / ms / 1e6, "hbm_frac": algo / ms / 1e6 / HBM_PEAK_GBS,
                         "surviving_TFLOPs": flops_surv / ms / 1e9}
    algo_step = 3 * comp + G * sum(M * case.K * 2 + M * case.N * 4 for M in (1, 8, 16))
    launch_ms = ev_ms / 3.0
    achieved = algo_step / 3.0 / launch_ms / 1e6
    out = {
        "metric": "compressed-weight HBM GB/s of the unified/pruned GEMM (decode regime, M<=16)",
        "value": 3 * comp / wall_ms / 1e6,
        "unit": "GB/s",
        "ms_per_step": wall_ms,
        "config": {"workload": "cfg4_decode_projections", "N": case.N, "K": case.K, "B": case.B,
                   "r_unify": case.r_unify, "r_prune": case.r_prune, "M": [1, 8, 16], "groups": G,
                   "distinct_matrices": ndist, "launches_per_step": 3,
                   "compressed_bytes_per_matrix": comp // G},
        "roofline": {"kernel": "k_stream_bf16<16>", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic_from_profiles("k_stream_bf16_cfg4"),
                     "algorithmic_bytes_per_launch": algo_step / 3.0, "avg_launch_ms": launch_ms},
        "per_M": per_M,
    }
    # yardstick: the dense bf16 GEMMs of the same shapes through torch (hipBLASLt), M = 16
    try:
        Wd = torch.stack([muw.muw_decode(layers[g % ndist]) for g in range(min(G, 32))])
        Xd = torch.stack(groups[16].Xs[:Wd.shape[0]])
        _, ms = time_steps(torch, lambda: torch.bmm(Xd, Wd.transpose(1, 2)), 10, 2)
        out["yardstick_dense_bf16_bmm_M16"] = {"groups": int(Wd.shape[0]), "ms": ms,
                                               "dense_weight_GBps": Wd.numel() * 2 / ms / 1e6}
        del Wd, Xd
    except Exception as e:  # a yardstick only
        log(f"[bench] dense yardstick skipped: {e}")

    if not args.no_cpu_baseline:
        from oracle import muw_oracle as oracle
        # the oracle as it stands: encode two of the distinct matrices, then repeat their
        # M = 1, 8, 16 GEMMs until about 10 s of CPU time have been spent
        Whats = []
        for g in range(min(2, len(host_W))):
            W64 = host_W[g].f64()
            n_u, n_p = oracle.counts(W64.size // case.B, case.r_unify, case.r_prune)
            Whats.append(oracle.encode(W64, case.B, n_u, n_p, oracle.STORE_BF16)[3].astype("float32"))
        passes, t0 = 0, time.perf_counter()
        while time.perf_counter() - t0 < 10.0:
            g = passes % len(Whats)
            for M in (1, 8, 16):
                oracle.gemm_f32in(host_X[(M, g)].f32(), Whats[g])
            passes += 1
        t_gemm = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": passes * 3 * (comp / G) / t_gemm / 1e9, "unit": "GB/s",
                               "cores": oracle.omp_threads(), "kind": "oracle",
                               "sample": f"{passes} passes of the oracle GEMM (fp64 accumulate, dense projected "
                                         f"weights) over 1 matrix at M=1,8,16, {t_gemm:.1f} s; rate counted in "
                                         "compressed-weight bytes like `value`"}
    return out


def bench_cfg5(args, torch, muw, synth, to_device):
    res = {}
    total_flops_surv, total_ms = 0.0, 0.0
    for which in ("up", "down"):
        case = synth.config5(2048, which)
        X, W = synth.make_linear(case)
        layer = muw.muw_encode(to_device(W), case.B, case.r_unify, case.r_prune)
        Xd = to_device(X)
        Y = torch.empty((case.M, case.N), dtype=torch.float32, device="cuda")
        _, ms = time_steps(torch, lambda: muw.muw_gemm(layer, Xd, out=Y), args.steps, args.warmup)
        surv = 2.0 * case.M * case.B * (layer.NB - layer.desc.n_pruned)
        dense = 2.0 * case.M * case.N * case.K
        res[which] = {"ms": ms, "surviving_TFLOPs": surv / ms / 1e9, "executed_dense_TFLOPs": dense / ms / 1e9}
        total_flops_surv += surv
        total_ms += ms
    return {"metric": "dense-equivalent TFLOP/s on surviving blocks (M=2048 MLP GEMMs)",
            "value": total_flops_surv / total_ms / 1e9, "unit": "TFLOP/s", "ms_per_step": total_ms,
            "config": {"workload": "cfg5_mlp_M2048"}, "per_gemm": res,
            "roofline": {"bound": "mfma", "achieved": total_flops_surv / total_ms / 1e9, "peak": MFMA_BF16_PEAK_TFLOPS,
                         "unit": "TFLOP/s", "frac": total_flops_surv / total_ms / 1e9 / MFMA_BF16_PEAK_TFLOPS,
                         "traffic": None}}


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures ONE GPU only (no collectives, no sharding); run with --gpus 1")
    import torch

    from paper_2106_08301_amd import binding as muw
    from paper_2106_08301_amd import synth
    from tests.gpu_util import to_device

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    torch.cuda.set_device(0)
    if args.workload == "cfg4":
        out = bench_cfg4(args, torch, muw, synth, to_device)
    else:
        out = bench_cfg5(args, torch, muw, synth, to_device)
    line = {"metric": out.pop("metric"), "value": out.pop("value"), "unit": out.pop("unit"), "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": out.pop("ms_per_step"),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
            "data": "synthetic", "config": out.pop("config")}
    line.update(out)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
