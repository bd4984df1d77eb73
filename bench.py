#!/usr/bin/env python3
"""Benchmark of the MergeComp hot path on one MI355X.

Workload (the benchmark's third configuration): ResNet-50-shaped gradients, 161 tensors,
25 557 032 fp32, merged into y = 1 group, W = 8 simulated workers resident on
the GPU.  One step = for each of EF-Sign and Top-k 1 %: one worker's
mc_compress of the whole model followed by one mc_decompress_sum over the W
payloads -- what one GPU does per iteration of the paper's Algorithm 1.  The
worker whose (gradient, state) buffers are compressed rotates every step, and
every worker draws a NEW gradient each time its turn comes (Algorithm 1:
g = stochasticGradient per iteration): it cycles over FRESH pre-generated
gradients, so the sparsifiers' thresholds move from call to call as they do in
training and the working set (W x FRESH x 102 MB of gradients plus W x 102 MB of
state per algorithm) is far larger than the 256 MB last-level cache.

value = fp32 gradient bytes pushed through compress + decompress per second
(2 algorithms x 4 D bytes per step / step time).  `roofline` is the dominant
kernel's algorithmic bytes per launch over its HIP-event time, against the
8 TB/s HBM peak, with the whole-call fractions beside it.  `cpu_baseline` is the
plain C oracle timed on this host.

Prints ONE JSON line.  Runs on one GPU only (--gpus above 1 exits).
"""
from __future__ import annotations

import argparse
import json
import os
import platform
import sys
import time
from concurrent.futures import ThreadPoolExecutor

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
# Whole-call algorithmic bytes per element (compress, decompress-sum) at kept fraction rho (the sparse payloads'
# directory, 4 bytes per 4096 elements, is left out: 0.001 bytes per element)
CALL_BYTES = {
    "efsign": (lambda rho: 12.125, lambda W, rho: W / 8.0 + 4.0), "topk": (lambda rho: 12.0 + 8.0 * rho, lambda W, rho: 4.0 + 8.0 * rho * W),
    "dgc": (lambda rho: 20.0 + 8.0 * rho, lambda W, rho: 4.0 + 8.0 * rho * W), "qsgd": (lambda rho: 13.0, lambda W, rho: W + 4.0),
    "terngrad": (lambda rho: 12.25, lambda W, rho: W / 4.0 + 4.0), "fp16": (lambda rho: 14.0, lambda W, rho: 2.0 * W + 4.0),
    # the four further schemes of the paper's Table 1
    "signsgd": (lambda rho: 4.125, lambda W, rho: W / 8.0 + 4.0), "signum": (lambda rho: 12.125, lambda W, rho: W / 8.0 + 4.0),
    "onebit": (lambda rho: 12.125, lambda W, rho: W / 8.0 + 4.0), "randk": (lambda rho: 12.0 + 8.0 * rho, lambda W, rho: 4.0 + 8.0 * rho * W),
}
SPARSE = ("topk", "dgc", "randk")

CPU_STEPS = 3          # steps of the oracle that the cpu_baseline leg times (about 10 s)
SETTLE_CALLS = 16      # calls per worker with which a sparsifier's context is brought to its steady state (set-up, untimed)
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic_resnet50.txt")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=64,
                    help="untimed steps; each worker (one compress per step, rotating over W) needs a handful of calls "
                         "before its error-feedback state and the sparsifiers' threshold hints have settled")
    ap.add_argument("--y", type=int, default=1, help="number of merged groups for the headline run")
    ap.add_argument("--fresh", type=int, default=3, help="pre-generated gradients that every worker cycles over (1: the same every call)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--no-curve", action="store_true", help="skip the compress-time-vs-y curve and the partition search fed from it")
    ap.add_argument("--no-layerwise", action="store_true",
                    help="skip the layer-wise comparison (y = number of tensors: one compress / decompress per tensor)")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the ResNet-101 (W = 16) and Mask R-CNN secondary entries")
    ap.add_argument("--no-extras", action="store_true", help="skip the static-gradient line and the cold-call timing")
    ap.add_argument("--algos", default=None, help="bench lines, comma separated (default: efsign,topk; efsign,topk-0.1 with --config 3)")
    ap.add_argument("--config", type=int, default=2, choices=[2, 3, 4],
                    help="benchmark configuration of the main run: 2 ResNet-50 (W = 8, the headline), 3 ResNet-101 (W = 16, Top-k 0.1 %%), "
                         "4 Mask R-CNN (W = 8); 3 and 4 are for profiling, the default run reports them under other_configs")
    ap.add_argument("--grad-layout", default="separate", choices=["separate", "views"],
                    help="separate: every gradient tensor its own allocation (a model's .grad tensors); views: the "
                         "tensors of a worker are views into one buffer (a bucketed gradient store)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run 10 plain device copies of 256 MiB (a kernel of known traffic, used to scale "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def algo_config(name):
    """(library algorithm name, kept fraction in ppm, sample ppm) of a bench line."""
    base = name.split("-")[0]
    ppm = 1000 if base == "dgc" or name.endswith("-0.1") else 10000       # the configuration's ratios: Top-k 1 %, DGC 0.1 %
    return base, ppm, (10000 if name == "dgc-sampled" else 0)


class AlgoBench:
    """Buffers and calls of one algorithm on a workload.  grads[w][v]: tensor list of worker w's v-th gradient."""

    def __init__(self, B, torch, name, numel, y, W, grads, settle=True, policy=None):
        self.name, self.W, self.y = name, W, y
        base, ratio_ppm, sample = algo_config(name)
        self.bounds = B.mc_partition(numel, y, B.MC_PART_EVEN_ELEMS if policy is None else policy)
        self.ctx = B.Context(base, numel, self.bounds, ratio_ppm=ratio_ppm, seed=1, dgc_sample_ppm=sample)
        dev = "cuda:0"
        self.V = len(grads[0])
        self.state = [[torch.zeros(self.ctx.state_bytes(j), dtype=torch.uint8, device=dev) for j in range(y)] for _ in range(W)]
        self.pay = [[torch.zeros(self.ctx.payload_bytes(j), dtype=torch.uint8, device=dev) for j in range(y)] for _ in range(W)]
        g0 = grads[0][0]
        if len(g0) > 1 and g0[0].data_ptr() + 4 * g0[0].numel() == g0[1].data_ptr():      # views of one packed buffer
            flat = torch.empty(sum(numel), dtype=torch.float32, device=dev)
            offs = np.concatenate([[0], np.cumsum(numel)])
            self.outs = [flat[offs[t]:offs[t + 1]] for t in range(len(numel))]
        else:
            self.outs = [torch.empty_like(t) for t in g0]
        b = self.bounds
        # address lists are marshalled once: the loop below measures the library, not Python
        self.grad_arr = [[[B.ptr_array(grads[w % len(grads)][v][b[j]:b[j + 1]]) for j in range(y)] for v in range(self.V)] for w in range(W)]
        self.out_arr = [B.ptr_array(self.outs[b[j]:b[j + 1]]) for j in range(y)]
        self.pay_arr = [(B.ptr_array([self.pay[w][j] for w in range(W)]), W) for j in range(y)]
        # ... and for the calls that take all groups at once
        self.grad_all = [[B.ptr_array(grads[w % len(grads)][v]) for v in range(self.V)] for w in range(W)]
        self.state_all = [B.ptr_array(self.state[w]) for w in range(W)] if self.ctx.cfg.use_ef else [None] * W
        self.pay_of = [B.ptr_array(self.pay[w]) for w in range(W)]
        self.pay_all = B.ptr_array([self.pay[w][j] for w in range(W) for j in range(y)])
        self.out_all = B.ptr_array(self.outs)
        self.it = 0
        self.turn = [0] * W            # how many gradients each worker has compressed: it takes number turn % V next
        # Every worker has a payload before the first decompress.  The sparsifiers also leave their start-up
        # behind here (the first calls of a context have no threshold to filter with and take the slow routes; the
        # filter margin then needs a dozen calls to settle), so that --warmup may be small.
        for rep in range(SETTLE_CALLS if base in SPARSE and settle else 1):
            for w in range(W):
                self.compress(w)

    def compress(self, w):
        v = self.turn[w] % self.V
        self.turn[w] += 1
        self.it += 1
        for j in range(self.y):
            self.ctx.mc_compress(j, w, self.it, self.grad_arr[w][v][j], self.state[w][j], self.pay[w][j])

    def decompress(self):
        for j in range(self.y):
            self.ctx.mc_decompress_sum(j, self.pay_arr[j][0], 1.0, self.out_arr[j])

    def compress_groups(self, w):
        v = self.turn[w] % self.V
        self.turn[w] += 1
        self.it += 1
        self.ctx.mc_compress_groups(w, self.it, self.grad_all[w][v], self.state_all[w], self.pay_of[w])

    def decompress_groups(self):
        self.ctx.mc_decompress_sum_groups(self.pay_all, self.W, 1.0, self.out_all)

    def step(self, i):
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


def timed_dist(torch, fn, reps, batches=25):
    """Seconds per call over `batches` runs of reps / batches calls each: (median, p10, p90) of the batch means.  The
    diagnostic per-algorithm figures should not carry a single host stall (the headline keeps the plain K-step bracket)."""
    per = max(1, reps // batches)
    xs = np.array([timed(torch, lambda i, b=b: fn(b * per + i), per) for b in range(batches)])
    return float(np.median(xs)), float(np.percentile(xs, 10)), float(np.percentile(xs, 90))


def call_entry(name, D, W, tc, td, tc_q=None, td_q=None):
    base, ppm, _ = algo_config(name)
    entry = {"compress_us": tc * 1e6, "decompress_sum_us": td * 1e6, "gradient_GBps": 4.0 * D / (tc + td) * 1e-9}
    if tc_q is not None:
        entry["compress_us_p10_p90"] = [tc_q[0] * 1e6, tc_q[1] * 1e6]
        entry["decompress_sum_us_p10_p90"] = [td_q[0] * 1e6, td_q[1] * 1e6]
    if base in CALL_BYTES:
        rho = ppm * 1e-6
        bc, bd = CALL_BYTES[base]
        algb = (bc(rho) + bd(W, rho)) * D
        entry["algorithmic_GBps"] = algb / (tc + td) * 1e-9
        entry["roofline_frac"] = entry["algorithmic_GBps"] / HBM_PEAK_GBS
    return entry


def measure_calls(torch, ab, reps=250):
    W = ab.W
    tc, c10, c90 = timed_dist(torch, lambda i: ab.compress(i % W), reps)
    td, d10, d90 = timed_dist(torch, lambda i: ab.decompress(), reps)
    return tc, td, (c10, c90), (d10, d90)


def device_grads(torch, flats, numel, layout):
    offs = np.concatenate([[0], np.cumsum(numel)])
    if layout == "views":
        bufs = [torch.from_numpy(f).to("cuda:0") for f in flats]
        return [[b[offs[t]:offs[t + 1]] for t in range(len(numel))] for b in bufs]
    return [[torch.from_numpy(f[offs[t]:offs[t + 1]]).to("cuda:0") for t in range(len(numel))] for f in flats]


def cpu_model_string():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return platform.processor() or "unknown"


def read_traffic():
    """HBM bytes per launch by kernel slot, as the profile summary script left them (rocprofv3 FETCH_SIZE / WRITE_SIZE, see
    profiles/); an empty dict if that file is not there."""
    out = {}
    try:
        for line in open(TRAFFIC_FILE):
            parts = line.split()
            if len(parts) >= 2 and not line.startswith("#"):
                out[parts[0]] = float(parts[1])
    except OSError:
        pass
    return out


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
    wl = WL.workload(args.config)
    numel = wl.numel.tolist()
    D, W = wl.total, wl.workers
    algos = (args.algos or ("efsign,topk-0.1" if args.config == 3 else "efsign,topk")).split(",")
    if args.config != 2:
        args.no_other_configs = True
    V = max(1, args.fresh)

    flats = [[WL.gradients_flat(wl, w, v) for v in range(V)] for w in range(W)]
    grads = [device_grads(torch, flats[w], numel, args.grad_layout) for w in range(W)]          # grads[w][v][tensor]

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
            fl = [np.random.default_rng([77, w, v]).standard_normal(int(D), dtype=np.float32) * np.float32(0.01) for v in range(V)]
            grads_even.append(device_grads(torch, fl, numel, "separate"))

    grads_shared = None
    if any(a.endswith("-shared") for a in algos):
        # half of every worker's gradient is a component common to all workers: their kept indices then largely coincide
        # (the decompress-sum adds up to W values into the same element instead of W different ones)
        grads_shared = [device_grads(torch, [WL.gradients_flat(wl, w, v, shared_fraction=0.5) for v in range(V)], numel, "separate")
                        for w in range(W)]

    def grads_for(a):
        return grads_even if a.endswith("-even") else grads_shared if a.endswith("-shared") else grads
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
    for a in algos:
        if algo_config(a)[0] in SPARSE and not algo_config(a)[2]:
            benches[a].ctx.mc_select_stats(reset=True)
    sec = timed(torch, step, args.steps)
    prof = benches[dom_algo].ctx.profile_read()[dom_kernel]
    benches[dom_algo].ctx.profile_enable(False)
    # which route the sparsifiers' exact selection took in the timed steps (the result is the same on all; the cost is not)
    select_routes = {}
    for a in algos:
        if algo_config(a)[0] in SPARSE and not algo_config(a)[2]:
            s = benches[a].ctx.mc_select_stats()
            select_routes[a] = {r: int(s[r]) for r in ("fast", "dense", "above", "refill")}
            select_routes[a]["keys_in_threshold_bin_last_call"] = int(s["last_bin_keys"])
            select_routes[a]["candidates_last_call"] = int(s["last_candidates"])
            select_routes[a]["filter_margin_halvings_last_call"] = int(s["margin_halvings"])
    kern_us = 1e3 * prof["total_ms"] / prof["launches"]
    n_group = max(benches[dom_algo].ctx.group_numel(j) for j in range(args.y))
    launches_per_step = prof["launches"] / args.steps
    alg_bytes = ALGO_BYTES[dom_kernel](D, W, algo_config(dom_algo)[1] * 1e-6) / launches_per_step
    achieved = alg_bytes / kern_us * 1e-3      # GB/s
    grad_bytes = 4.0 * D * len(algos)
    value = grad_bytes / sec * 1e-9

    per_algo = {}
    for a in algos:
        tc, td, cq, dq = measure_calls(torch, benches[a])
        per_algo[a] = call_entry(a, D, W, tc, td, cq, dq)

    # ---- what the first call of a context costs, and the same calls on a gradient that never changes ------------------
    extras = None
    if not args.no_extras:
        extras = {"cold_call_us": {}, "static_gradient": {}}
        for a in algos:
            fresh_ctx = AlgoBench(B, torch, a, numel, args.y, 1, [grads_for(a)[0][:1]], settle=False)      # one worker, one compress done
            torch.cuda.synchronize()
            del fresh_ctx.ctx
            cold = []
            for rep in range(3):
                ab = AlgoBench.__new__(AlgoBench)
                base, ppm, sample = algo_config(a)
                bounds = B.mc_partition(numel, args.y, B.MC_PART_EVEN_ELEMS)
                ctx = B.Context(base, numel, bounds, ratio_ppm=ppm, seed=1, dgc_sample_ppm=sample)
                st = [torch.zeros(ctx.state_bytes(j), dtype=torch.uint8, device="cuda:0") for j in range(args.y)]
                py = [torch.zeros(ctx.payload_bytes(j), dtype=torch.uint8, device="cuda:0") for j in range(args.y)]
                ga = [B.ptr_array(grads_for(a)[0][0][bounds[j]:bounds[j + 1]]) for j in range(args.y)]
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for j in range(args.y):
                    ctx.mc_compress(j, 0, 1, ga[j], st[j], py[j])
                torch.cuda.synchronize()
                cold.append((time.perf_counter() - t0) * 1e6)
                ctx.close()
            extras["cold_call_us"][a] = float(np.median(cold))
            if algo_config(a)[0] in SPARSE and V > 1:
                sb = AlgoBench(B, torch, a, numel, args.y, W, [g[:1] for g in grads_for(a)])
                for i in range(2 * W):
                    sb.step(i)
                tc, td, cq, dq = measure_calls(torch, sb, 100)
                extras["static_gradient"][a] = call_entry(a, D, W, tc, td)
                sb.close()
                del sb
                torch.cuda.empty_cache()

    # ---- compress time vs number of groups (Lemma 2: sum_i h(x_i) = y B_h + gamma_h D) -------------
    curve = None
    search = None
    if not args.no_curve:
        curve = {}
        for a in algos:
            pts = []
            for y in wl.ys:
                ab = benches[a] if y == args.y else AlgoBench(B, torch, a, numel, y, W, grads_for(a))
                if ab is not benches[a]:
                    for i in range(4 * W):            # let the new context's state and hints settle
                        ab.compress(i % W)
                t = timed(torch, lambda i: ab.compress(i % W), 40)
                pts.append((y, t * 1e6))
                if ab is not benches[a]:
                    ab.close()
                    del ab
                    torch.cuda.empty_cache()
            ys = np.array([p[0] for p in pts], float)
            ts = np.array([p[1] for p in pts], float)
            A = np.stack([ys, np.ones_like(ys)], 1)
            (bh, c0), *_ = np.linalg.lstsq(A, ts, rcond=None)
            # the paper's naive partition (even by tensor count, Section 5.2) at the largest y: by Lemma 2 the total is the same
            yc = int(max(wl.ys))
            ab = AlgoBench(B, torch, a, numel, yc, W, grads_for(a), policy=B.MC_PART_EVEN_COUNT)
            for i in range(4 * W):
                ab.compress(i % W)
            t_count = timed(torch, lambda i: ab.compress(i % W), 40) * 1e6
            ab.close()
            del ab
            torch.cuda.empty_cache()
            curve[a] = {"y": [int(v) for v in ys], "compress_us": [float(v) for v in ts], "B_h_us": float(bh),
                        "gamma_h_D_us": float(c0), "inv_gamma_h_GBps": float(4.0 * D / c0 * 1e-3) if c0 > 0 else None,
                        "even_count_partition": {"y": yc, "compress_us": float(t_count)}}
        # ---- Algorithm 2 fed with the h(x) just measured ---------------------------------------------------------
        search = {}
        for a in algos:
            base, ppm, _ = algo_config(a)
            if base not in CALL_BYTES:
                continue
            bwd, mp = WL.iteration_timeline(numel, max(curve[a]["B_h_us"], 0.0) * 1e-6, max(curve[a]["gamma_h_D_us"], 0.0) * 1e-6 / D,
                                            WL.sent_bytes_per_elem(base, ppm))
            model = B.McTimeModel(*mp)
            Y, alpha = 4, 0.01
            bounds, F = B.mc_partition_search(numel, bwd, model, Y, alpha)
            y_star = len(bounds) - 1
            even_e = B.mc_partition(numel, y_star, B.MC_PART_EVEN_ELEMS)
            even_c = B.mc_partition(numel, y_star, B.MC_PART_EVEN_COUNT)
            search[a] = {"Y": Y, "alpha": alpha, "y": y_star, "bounds": bounds, "F_ms": F * 1e3,
                         "F_even_elems_ms": B.mc_partition_cost(numel, bwd, model, even_e) * 1e3,
                         "F_even_count_ms": B.mc_partition_cost(numel, bwd, model, even_c) * 1e3,
                         "F_one_group_ms": B.mc_partition_cost(numel, bwd, model, [0, len(numel)]) * 1e3,
                         "model": "h(x) as measured here; iteration 64 ms and 66 ms per 102 MB of fp32 over 2 x V100 PCIe as in "
                                  "Section 3.3 of the paper, scaled to the payload's bytes; 50 us per message"}

    # ---- layer-wise compression (Section 3: one encode and one decode per tensor) against merged ---------
    layerwise = None
    if not args.no_layerwise:
        layerwise = {}
        N = len(numel)
        for a in algos:
            lb = AlgoBench(B, torch, a, numel, N, W, grads_for(a))
            for i in range(2 * W):
                lb.compress(i % W)
            tc = timed(torch, lambda i: lb.compress(i % W), 10)
            td = timed(torch, lambda i: lb.decompress(), 10)
            # the same 161 compressions / decompressions looped over inside the library: no Python between them
            tcg = timed(torch, lambda i: lb.compress_groups(i % W), 10)
            tdg = timed(torch, lambda i: lb.decompress_groups(), 10)
            lb.close()
            del lb
            torch.cuda.empty_cache()
            merged = per_algo[a]["compress_us"] + per_algo[a]["decompress_sum_us"]
            layerwise[a] = {"groups": N, "compress_us": tc * 1e6, "decompress_sum_us": td * 1e6,
                            "merged_over_layerwise_speedup": (tc + td) * 1e6 / merged,
                            "looped_in_the_library": {"compress_us": tcg * 1e6, "decompress_sum_us": tdg * 1e6,
                                                      "merged_over_layerwise_speedup": (tcg + tdg) * 1e6 / merged}}

    for b in benches.values():
        b.close()
    benches.clear()
    del grads, grads_even, grads_shared
    torch.cuda.empty_cache()

    # ---- the other two large configurations: ResNet-101 with W = 16, Mask R-CNN with W = 8 --------------------------------
    others = None
    if not args.no_other_configs:
        others = {}
        for cfg, lines in ((3, ("efsign", "topk-0.1")), (4, ("efsign", "topk"))):
            w2 = WL.workload(cfg)
            numel2, D2, W2 = w2.numel.tolist(), w2.total, w2.workers
            distinct = min(W2, 4)              # four distinct workers' gradients, shared round-robin by the W workers (set-up time)
            fl = [WL.gradients_flat(w2, w, 0) for w in range(distinct)]
            g2 = [device_grads(torch, [fl[w]], numel2, "separate") for w in range(distinct)]
            entry = {"workload": f"{w2.name}-shaped gradients, {len(numel2)} tensors, {D2} fp32", "workers": W2, "y": 1,
                     "gradients": f"{distinct} distinct workers' gradients, static"}
            for a in lines:
                ab = AlgoBench(B, torch, a, numel2, 1, W2, g2)
                for i in range(2 * W2):
                    ab.step(i)
                tc, td, cq, dq = measure_calls(torch, ab, 100)
                entry[a] = call_entry(a, D2, W2, tc, td, cq, dq)
                ab.close()
                del ab
                torch.cuda.empty_cache()
            others[w2.name] = entry
            del g2, fl
            torch.cuda.empty_cache()

    # ---- the oracle on this host's cores -----------------------------------------------------------
    cpu = None
    if not args.no_cpu:
        from oracle import oracle as O
        T = os.cpu_count() or 1

        def ocfg_of(a):
            base, ppm, sample = algo_config(a)
            return O.Config(B.ALGO_IDS[base], ratio_ppm=ppm, seed=1, use_ef=0 if base == "signsgd" else 1, dgc_sample_ppm=sample)
        t_cpu = 0.0
        for a in algos:
            ocfg = ocfg_of(a)
            st = O.new_state(ocfg, D)
            t0 = time.perf_counter()
            for it in range(CPU_STEPS):          # the state carries the error feedback from step to step
                pay, _ = O.compress(ocfg, flats[0][it % V], st, it=it)
                O.decompress_sum([pay] * W, D, 1.0)
            t_cpu += time.perf_counter() - t0
        # T threads over the independent units of one step of all W workers: the W compress calls side by side (the C
        # routines release the interpreter lock), then the one decompress-sum, per algorithm; no change to a unit's code
        t_par, units = 0.0, 0
        with ThreadPoolExecutor(max_workers=T) as pool:
            for a in algos:
                ocfg = ocfg_of(a)
                sts = [O.new_state(ocfg, D) for _ in range(W)]
                t0 = time.perf_counter()
                pays = list(pool.map(lambda w: O.compress(ocfg, flats[w][0], sts[w], worker=w, it=0)[0], range(W)))
                O.decompress_sum(pays, D, 1.0)
                t_par += time.perf_counter() - t0
                units += W + 1
        cpu = {"value": CPU_STEPS * grad_bytes / t_cpu * 1e-9, "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"{CPU_STEPS} full steps on the same ResNet-50-shaped input: worker 0's compress and a decompress-sum over "
                         f"{W} copies of its payload, for each of {'+'.join(algos)}; {t_cpu:.1f} s single-threaded",
               "host_cpus": T, "cpu_model": cpu_model_string(),
               "threads": {"cores": min(T, W), "value": W * grad_bytes / t_par * 1e-9, "unit": "GB/s",
                           "sample": f"one step of all {W} workers per algorithm: the {W} compress calls on {min(T, W)} threads, then one "
                                     f"decompress-sum over their payloads; {units} units, {t_par:.1f} s"}}

    traffic = read_traffic() if args.config == 2 else {}          # the file holds the ResNet-50 run's counters
    result = {
        "metric": "compress+decompress GB/s of fp32 gradient (EF-Sign, Top-k 1%) vs HBM peak",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}-shaped gradients, {len(numel)} tensors, {D} fp32, "
                               + ("Student-t(3) values, " if args.config == 4 else "") + "per-tensor std log-uniform [1e-4,1e-1]",
                   "y": args.y, "workers": W, "grad_layout": args.grad_layout, "algorithms": algos, "topk_ratio_ppm": 1000 if args.config == 3 else 10000,
                   "gradients_per_worker": V,
                   "step": "per algorithm: one worker's mc_compress of its next gradient + one mc_decompress_sum over W payloads"},
        "roofline": {"bound": "hbm", "kernel": f"{dom_algo}:{dom_kernel}", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic.get(dom_kernel),
                     "algorithmic_bytes_per_launch": alg_bytes, "avg_launch_us": kern_us,
                     "elements_per_launch": n_group,
                     "whole_call_frac": {a: per_algo[a].get("roofline_frac") for a in algos},
                     "note": "frac is the dominant kernel's; whole_call_frac is compress + decompress-sum of each algorithm, "
                             "all their kernels and the gaps between them included, against the same peak"},
        "cpu_baseline": cpu,
        "per_algo": per_algo,
        "select_routes": select_routes,
        "kernels_us_per_step": {k: round(v["us_per_step"], 2) for k, v in sorted(kernels.items())},
        "extras": extras,
        "compress_time_vs_y": curve,
        "partition_search": search,
        "layerwise_vs_merged": layerwise,
        "other_configs": others,
    }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
