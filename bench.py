#!/usr/bin/env python3
"""Benchmark of the MergeComp hot path on one MI355X.

Workload (the benchmark's third configuration): ResNet-50-shaped gradients, 161 tensors,
25 557 032 fp32, merged into y = 1 group, W = 8 simulated workers resident on
the GPU.  One step = for each of EF-Sign and Top-k 1 %: one worker's
mc_compress of the whole model followed by one mc_decompress_sum over the W
payloads -- what one GPU does per iteration of the paper's Algorithm 1.  The
worker whose (gradient, state) buffers are compressed rotates every step, so
the working set (W x 204 MB per algorithm) is far larger than the 256 MB
last-level cache and the reads really come from HBM.

value = fp32 gradient bytes pushed through compress + decompress per second
(2 algorithms x 4 D bytes per step / step time).  `roofline` is the dominant
kernel's algorithmic bytes per launch over its HIP-event time, against the
8 TB/s HBM peak.  `cpu_baseline` is the plain C oracle timed on this host.

Prints ONE JSON line.  Runs on one GPU only (--gpus above 1 exits).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# Algorithmic HBM bytes per element of one launch (each operand touched once).
ALGO_BYTES = {
    "efsign_compress": lambda n, W, rho: 12.125 * n,            # read g, read p_prev, write p, 1 bit
    "sparse_accum": lambda n, W, rho: 12.0 * n,                 # read g, read e, write p
    "dense_decompress": lambda n, W, rho: (W / 8.0 + 4.0) * n,  # W sign planes in, fp32 out
    "sparse_decompress": lambda n, W, rho: (4.0 + 8.0 * rho * W) * n,
}
# Whole-call algorithmic bytes per element (compress, decompress-sum): Top-k 1 %, DGC 0.1 %
CALL_BYTES = {
    "efsign": (12.125, lambda W: W / 8.0 + 4.0), "topk": (12.08, lambda W: 4.0 + 0.08 * W),
    "dgc": (20.008, lambda W: 4.0 + 0.008 * W), "qsgd": (13.0, lambda W: W + 4.0),
    "terngrad": (12.25, lambda W: W / 4.0 + 4.0), "fp16": (14.0, lambda W: 2.0 * W + 4.0),
    # the four further schemes of the paper's Table 1 (Rand-k 1 %)
    "signsgd": (4.125, lambda W: W / 8.0 + 4.0), "signum": (12.125, lambda W: W / 8.0 + 4.0),
    "onebit": (12.125, lambda W: W / 8.0 + 4.0), "randk": (12.08, lambda W: 4.0 + 0.08 * W),
    # DGC 0.1 % with the threshold taken from a 1 % sample (about k entries kept, room for 2k)
    "dgc-sampled": (20.008, lambda W: 4.0 + 0.008 * W),
    # Top-k 1 % on tensors of one scale (`topk-even`: candidates spread over every tile)
    "topk-even": (12.08, lambda W: 4.0 + 0.08 * W),
}

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (see profiles/); None = not measured
MEASURED_TRAFFIC = {        # profiles/bench_resnet50_efsign_topk.txt, read + write, scaled by the copy calibration
    "efsign_compress": 313.58e6, "sparse_accum": 321.69e6, "dense_decompress": 129.23e6, "sparse_decompress": 136.86e6,
}


CPU_STEPS = 3          # steps of the oracle that the cpu_baseline leg times (about 10 s)
SETTLE_CALLS = 16      # calls per worker with which a sparsifier's context is brought to its steady state (set-up, untimed)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=64,
                    help="untimed steps; each worker (one compress per step, rotating over W) needs a handful of calls "
                         "before its error-feedback state and the sparsifiers' threshold hints have settled")
    ap.add_argument("--y", type=int, default=1, help="number of merged groups for the headline run")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--no-curve", action="store_true", help="skip the compress-time-vs-y curve")
    ap.add_argument("--no-layerwise", action="store_true",
                    help="skip the layer-wise comparison (y = number of tensors: one compress / decompress per tensor)")
    ap.add_argument("--algos", default="efsign,topk")
    ap.add_argument("--grad-layout", default="separate", choices=["separate", "views"],
                    help="separate: every gradient tensor its own allocation (a model's .grad tensors); views: the "
                         "tensors of a worker are views into one buffer (a bucketed gradient store)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run 10 plain device copies of 256 MiB (a kernel of known traffic, used to scale "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


class AlgoBench:
    """Buffers and calls of one algorithm on the workload."""

    def __init__(self, B, torch, name, numel, y, W, grads, settle=True):
        self.name, self.W, self.y = name, W, y
        ratio_ppm = 1000 if name.startswith("dgc") else 10000          # the configuration's ratios: Top-k 1 %, DGC 0.1 %
        self.bounds = B.mc_partition(numel, y, B.MC_PART_EVEN_ELEMS)
        self.ctx = B.Context(name.split("-")[0], numel, self.bounds, ratio_ppm=ratio_ppm, seed=1,
                             dgc_sample_ppm=10000 if name == "dgc-sampled" else 0)
        dev = "cuda:0"
        self.grads = grads
        self.state = [[torch.zeros(self.ctx.state_bytes(j), dtype=torch.uint8, device=dev) for j in range(y)] for _ in range(W)]
        self.pay = [[torch.zeros(self.ctx.payload_bytes(j), dtype=torch.uint8, device=dev) for j in range(y)] for _ in range(W)]
        if grads[0][0].data_ptr() + 4 * grads[0][0].numel() == grads[0][1].data_ptr():      # views of one packed buffer
            flat = torch.empty(sum(numel), dtype=torch.float32, device=dev)
            offs = np.concatenate([[0], np.cumsum(numel)])
            self.outs = [flat[offs[t]:offs[t + 1]] for t in range(len(numel))]
        else:
            self.outs = [torch.empty_like(t) for t in grads[0]]
        b = self.bounds
        # address lists are marshalled once: the loop below measures the library, not Python
        self.grad_arr = [[B.ptr_array(grads[w][b[j]:b[j + 1]]) for j in range(y)] for w in range(W)]
        self.out_arr = [B.ptr_array(self.outs[b[j]:b[j + 1]]) for j in range(y)]
        self.pay_arr = [(B.ptr_array([self.pay[w][j] for w in range(W)]), W) for j in range(y)]
        self.it = 0
        # Every worker has a payload before the first decompress.  The sparsifiers also leave their start-up
        # behind here (the first calls of a context have no threshold to filter with and take the slow routes; the
        # filter margin then needs a dozen calls to settle), so that --warmup may be small.
        for rep in range(SETTLE_CALLS if name.split("-")[0] in ("topk", "dgc", "randk") and settle else 1):
            self.it += 1 if rep else 0
            for w in range(W):
                self.compress(w)

    def compress(self, w):
        for j in range(self.y):
            self.ctx.mc_compress(j, w, self.it, self.grad_arr[w][j], self.state[w][j], self.pay[w][j])

    def decompress(self):
        for j in range(self.y):
            self.ctx.mc_decompress_sum(j, self.pay_arr[j][0], 1.0, self.out_arr[j])

    def step(self, i):
        self.it += 1
        self.compress(i % self.W)
        self.decompress()

    def close(self):
        self.ctx.close()


def timed(torch, fn, reps):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(reps):
        fn(i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / reps


def timed_median(torch, fn, reps, batches=5):
    """Seconds per call as the median over `batches` runs of reps / batches calls each: the diagnostic per-algorithm
    figures should not carry a single host stall (the headline keeps the plain K-step bracket)."""
    per = max(1, reps // batches)
    return float(np.median([timed(torch, lambda i, b=b: fn(b * per + i), per) for b in range(batches)]))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (each GPU is one worker; nothing in the path crosses GPUs); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2103_15195_amd import binding as B
    from paper_2103_15195_amd import workloads as WL

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    B.lib()          # fails loudly if the HIP library has not been built
    wl = WL.workload(2)
    numel = wl.numel.tolist()
    D, W = wl.total, wl.workers
    algos = args.algos.split(",")

    flats = [WL.gradients_flat(wl, w, 0) for w in range(W)]
    offs = np.concatenate([[0], np.cumsum(numel)])
    if args.grad_layout == "views":
        bufs = [torch.from_numpy(f).to("cuda:0") for f in flats]
        grads = [[b[offs[t]:offs[t + 1]] for t in range(len(numel))] for b in bufs]
    else:
        grads = [[torch.from_numpy(f[offs[t]:offs[t + 1]]).to("cuda:0") for t in range(len(numel))] for f in flats]

    if args.calibrate_copy:
        src = torch.ones(1 << 26, dtype=torch.float32, device="cuda:0")      # 256 MiB in, 256 MiB out per copy
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    grads_even = None
    if any(a.endswith("-even") for a in algos):
        # all tensors of one scale: under error feedback every element's |p| creeps up to the threshold, and the
        # sparsifiers' candidates spread evenly over the tiles instead of clustering in the tensors of large scale
        grads_even = []
        for w in range(W):
            f = np.random.default_rng([77, w]).standard_normal(int(D), dtype=np.float32) * np.float32(0.01)
            grads_even.append([torch.from_numpy(f[offs[t]:offs[t + 1]]).to("cuda:0") for t in range(len(numel))])
    def grads_for(a):
        return grads_even if a.endswith("-even") else grads
    benches = {a: AlgoBench(B, torch, a, numel, args.y, W, grads_for(a)) for a in algos}

    def step(i):
        for a in algos:
            benches[a].step(i)

    # ---- per-kernel profile (outside the timed region): find the dominant kernel -----------------
    for i in range(args.warmup):
        step(i)
    kernels = {}
    for a in algos:
        benches[a].ctx.profile_reset()
        benches[a].ctx.profile_enable(True, all_kernels=True)
    for i in range(16):
        step(i)
    for a in algos:
        for k, v in benches[a].ctx.profile_read().items():
            kernels[f"{a}:{k}"] = {"launches_per_step": v["launches"] / 16.0, "us_per_step": 1e3 * v["total_ms"] / 16.0}
        benches[a].ctx.profile_enable(False)
        benches[a].ctx.profile_reset()
    dom_key = max((k for k in kernels if k.split(":")[1] in ALGO_BYTES), key=lambda k: kernels[k]["us_per_step"])
    dom_algo, dom_kernel = dom_key.split(":")

    # ---- the timed region: exactly K steps; HIP events only around the dominant kernel -----------
    benches[dom_algo].ctx.profile_enable_only(dom_kernel)
    for i in range(4):
        step(i)
    benches[dom_algo].ctx.profile_reset()
    sec = timed(torch, step, args.steps)
    prof = benches[dom_algo].ctx.profile_read()[dom_kernel]
    benches[dom_algo].ctx.profile_enable(False)
    kern_us = 1e3 * prof["total_ms"] / prof["launches"]
    n_group = max(benches[dom_algo].ctx.group_numel(j) for j in range(args.y))
    launches_per_step = prof["launches"] / args.steps
    alg_bytes = ALGO_BYTES[dom_kernel](D, W, 0.01) / launches_per_step
    achieved = alg_bytes / kern_us * 1e-3      # GB/s
    grad_bytes = 4.0 * D * len(algos)
    value = grad_bytes / sec * 1e-9

    per_algo = {}
    for a in algos:
        tc = timed_median(torch, lambda i: (setattr(benches[a], "it", benches[a].it + 1), benches[a].compress(i % W)), 250)
        td = timed_median(torch, lambda i: benches[a].decompress(), 250)
        bc, bd = CALL_BYTES.get(a, (None, None))
        entry = {"compress_us": tc * 1e6, "decompress_sum_us": td * 1e6, "gradient_GBps": 4.0 * D / (tc + td) * 1e-9}
        if bc is not None:
            algb = (bc + bd(W)) * D
            entry["algorithmic_GBps"] = algb / (tc + td) * 1e-9
            entry["roofline_frac"] = entry["algorithmic_GBps"] / HBM_PEAK_GBS
        per_algo[a] = entry

    # ---- compress time vs number of groups (Lemma 2: sum_i h(x_i) = y B_h + gamma_h D) -------------
    curve = None
    if not args.no_curve:
        curve = {}
        for a in algos:
            pts = []
            for y in wl.ys:
                ab = benches[a] if y == args.y else AlgoBench(B, torch, a, numel, y, W, grads_for(a))
                if ab is not benches[a]:
                    for i in range(8 * W):            # let the new context's state and hints settle
                        ab.it += 1
                        ab.compress(i % W)
                t = timed(torch, lambda i: (setattr(ab, "it", ab.it + 1), ab.compress(i % W)), 40)
                pts.append((y, t * 1e6))
                if ab is not benches[a]:
                    ab.close()
                    del ab
                    torch.cuda.empty_cache()
            ys = np.array([p[0] for p in pts], float)
            ts = np.array([p[1] for p in pts], float)
            A = np.stack([ys, np.ones_like(ys)], 1)
            (bh, c0), *_ = np.linalg.lstsq(A, ts, rcond=None)
            curve[a] = {"y": [int(v) for v in ys], "compress_us": [float(v) for v in ts], "B_h_us": float(bh),
                        "gamma_h_D_us": float(c0), "inv_gamma_h_GBps": float(4.0 * D / c0 * 1e-3) if c0 > 0 else None}

    # ---- layer-wise compression (Section 3: one encode and one decode per tensor) against merged ---------
    layerwise = None
    if not args.no_layerwise:
        layerwise = {}
        N = len(numel)
        for a in algos:
            lb = AlgoBench(B, torch, a, numel, N, W, grads_for(a))
            for i in range(4 * W):
                lb.it += 1
                lb.compress(i % W)
            tc = timed(torch, lambda i: (setattr(lb, "it", lb.it + 1), lb.compress(i % W)), 10)
            td = timed(torch, lambda i: lb.decompress(), 10)
            lb.close()
            del lb
            torch.cuda.empty_cache()
            merged = per_algo[a]["compress_us"] + per_algo[a]["decompress_sum_us"]
            layerwise[a] = {"groups": N, "compress_us": tc * 1e6, "decompress_sum_us": td * 1e6,
                            "merged_over_layerwise_speedup": (tc + td) * 1e6 / merged}

    # ---- the oracle on this host's cores -----------------------------------------------------------
    cpu = None
    if not args.no_cpu:
        from oracle import oracle as O
        t_cpu = 0.0
        for a in algos:
            ocfg = O.Config(B.ALGO_IDS[a.split("-")[0]], ratio_ppm=1000 if a.startswith("dgc") else 10000, seed=1,
                            use_ef=0 if a == "signsgd" else 1, dgc_sample_ppm=10000 if a == "dgc-sampled" else 0)
            st = O.new_state(ocfg, D)
            t0 = time.perf_counter()
            for it in range(CPU_STEPS):          # the state carries the error feedback from step to step
                pay, _ = O.compress(ocfg, flats[0], st, it=it)
                O.decompress_sum([pay] * W, D, 1.0)
            t_cpu += time.perf_counter() - t0
        cpu = {"value": CPU_STEPS * grad_bytes / t_cpu * 1e-9, "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"{CPU_STEPS} full steps on the same ResNet-50-shaped input: worker 0's compress and a decompress-sum over "
                         f"{W} copies of its payload, for each of {'+'.join(algos)}; {t_cpu:.1f} s single-threaded",
               "host_cpus": os.cpu_count()}

    result = {
        "metric": "compress+decompress GB/s of fp32 gradient (EF-Sign, Top-k 1%) vs HBM peak",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "resnet50-shaped gradients, 161 tensors, 25557032 fp32, per-tensor std log-uniform [1e-4,1e-1]",
                   "y": args.y, "workers": W, "grad_layout": args.grad_layout, "algorithms": algos, "topk_ratio_ppm": 10000,
                   "step": "per algorithm: one worker's mc_compress + one mc_decompress_sum over W payloads"},
        "roofline": {"bound": "hbm", "kernel": f"{dom_algo}:{dom_kernel}", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC.get(dom_kernel),
                     "algorithmic_bytes_per_launch": alg_bytes, "avg_launch_us": kern_us,
                     "elements_per_launch": n_group},
        "cpu_baseline": cpu,
        "per_algo": per_algo,
        "kernels_us_per_step": {k: round(v["us_per_step"], 2) for k, v in sorted(kernels.items())},
        "compress_time_vs_y": curve,
        "layerwise_vs_merged": layerwise,
    }
    for b in benches.values():
        b.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
