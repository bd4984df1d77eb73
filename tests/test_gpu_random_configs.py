"""GPU-vs-oracle parity on seeded random configurations: tensor lists (empty, tiny, around multiples of the
1024-element chunk, large), partitions, worker counts, algorithms with their parameters, buffer layouts and value
distributions (normal, heavy-tailed, many ties and zeros, mostly zeros, one extreme scale).  Every case runs the full
protocol of the other parity tests (payload, residual and aggregate bit for bit)."""
import numpy as np
import pytest

import harness as H

pytestmark = pytest.mark.gpu

ALGOS = ["efsign", "topk", "dgc", "qsgd", "terngrad", "fp16", "signsgd", "signum", "onebit", "randk"]
CASES_PER_BLOCK = 30


def random_case(block, case):
    rng = np.random.default_rng([20210325, block, case])
    nt = int(rng.integers(1, 40))
    numel = []
    for kind in rng.integers(0, 5, nt):
        if kind == 0:
            numel.append(int(rng.integers(0, 3)))
        elif kind == 1:
            numel.append(int(rng.integers(1, 70)))
        elif kind == 2:
            numel.append(int(1024 * rng.integers(1, 9) + rng.integers(-2, 3)))
        elif kind == 3:
            numel.append(int(rng.integers(1, 20000)))
        else:
            numel.append(int(rng.integers(1, 300000)) if rng.random() < 0.3 else int(rng.integers(1, 5000)))
    if sum(numel) == 0:
        numel[0] = 5
    total = sum(numel)
    algo = ALGOS[int(rng.integers(0, len(ALGOS)))]
    cfg = dict(ratio_ppm=int(10 ** rng.uniform(0, 6)), seed=int(rng.integers(0, 2 ** 63)))
    if algo == "dgc" and rng.random() < 0.4:
        cfg["dgc_sample_ppm"] = int(10 ** rng.uniform(3, 6))
    if algo == "qsgd":
        cfg["qsgd_bits"] = int(rng.integers(2, 9))
    if algo in ("topk", "qsgd", "terngrad", "efsign", "fp16", "onebit") and rng.random() < 0.2:
        cfg["use_ef"] = 0
    y = int(rng.integers(1, min(4, nt) + 1))
    W = int(rng.choice([1, 2, 3, 5, 8, 9, 17]))
    values = int(rng.integers(0, 5))

    def grads(w, it):
        r = np.random.default_rng([20210325, block, case, w, it])
        if values == 0:
            return r.standard_normal(total, dtype=np.float32) * np.float32(0.01)
        if values == 1:
            return (r.standard_normal(total) * np.exp(3 * r.standard_normal(total))).astype(np.float32)
        if values == 2:
            return np.round(r.standard_normal(total) * 2).astype(np.float32)
        if values == 3:
            return (r.standard_normal(total) * (r.random(total) < 0.05)).astype(np.float32)
        return r.standard_normal(total, dtype=np.float32) * np.float32(10.0 ** r.integers(-30, 30))

    return dict(numel=numel, algo=algo, y=y, W=W, iters=int(rng.integers(1, 4)), grads_fn=grads,
                layout=str(rng.choice(["separate", "flat", "misaligned"])), alpha=float(rng.choice([1.0, 0.5, 1.0 / W])), **cfg)


@pytest.mark.parametrize("block", range(4))
def test_random_configurations(block):
    for case in range(CASES_PER_BLOCK):
        c = random_case(block, case)
        print(f"[block {block} case {case}] {c['algo']} y={c['y']} W={c['W']} iters={c['iters']} layout={c['layout']} "
              f"tensors={len(c['numel'])} total={sum(c['numel'])} " + " ".join(f"{k}={v}" for k, v in c.items()
                                                                              if k in ("ratio_ppm", "dgc_sample_ppm", "qsgd_bits", "use_ef")), flush=True)
        numel, algo, y, W, iters, grads_fn = (c.pop(k) for k in ("numel", "algo", "y", "W", "iters", "grads_fn"))
        H.run_parity(numel, algo, y, W, iters, grads_fn, **c)
