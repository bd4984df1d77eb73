"""Shared driver of the GPU-vs-oracle parity tests (not collected by pytest).

The HIP path is always reached through the C ABI (paper_2103_15195_amd.binding);
the expected values always come from oracle/ run on the same seeded inputs.

Bar: bit-exact packed codes, indices, sparsifier values and
residuals; group scalars (EF-Sign scale, QSGD norm) within 1e-6 relative, TernGrad
max bit-exact; aggregated sums within 1e-6 relative to sum_w |d_w| -- the tests
assert the stricter bit equality for the sums, because both sides add the same
fp32 terms in the same worker order.

Scalars and codes.  QSGD / TernGrad codes and every residual depend on the group
scalar (OneBit: on its two class means).  The oracle first runs on its own; if its scalar has the same bits as the
GPU's (the normal case: both accumulate in fp64) everything must match bit for
bit.  If the scalars differ within the 1e-6 bar, the oracle's encode step is
repeated with the GPU's scalar as input and must then match bit for bit; this is
counted in Stats.conditional.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence

import numpy as np
import torch

from oracle import oracle as O
from paper_2103_15195_amd import binding as B
from paper_2103_15195_amd import workloads as WL

ALGOS = {"efsign": 1, "topk": 2, "dgc": 3, "qsgd": 4, "terngrad": 5, "fp16": 6,
         "signsgd": 7, "signum": 8, "onebit": 9, "randk": 10}
DEV = "cuda:0"


@dataclass
class Stats:
    compress_checks: int = 0
    decompress_checks: int = 0
    conditional: int = 0
    notes: List[str] = field(default_factory=list)


def u32(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a).view(np.uint32)


def same_bits(a: np.ndarray, b: np.ndarray) -> bool:
    return a.shape == b.shape and np.array_equal(u32(a), u32(b))


def device_tensors(flat: np.ndarray, numel: Sequence[int], layout: str = "separate") -> List[torch.Tensor]:
    """The tensor list of one worker on the GPU.
    separate   : every tensor its own allocation (what a model's .grad tensors look like)
    flat       : views into one buffer
    misaligned : views into one buffer shifted by one element (4-byte but not 16-byte aligned)"""
    offs = np.concatenate([[0], np.cumsum(numel)]).astype(np.int64)
    if layout == "separate":
        return [torch.from_numpy(np.ascontiguousarray(flat[offs[t]:offs[t + 1]])).to(DEV) for t in range(len(numel))]
    shift = 1 if layout == "misaligned" else 0
    buf = torch.zeros(int(offs[-1]) + shift + 4, dtype=torch.float32, device=DEV)
    buf[shift:shift + int(offs[-1])] = torch.from_numpy(flat).to(DEV)
    return [buf[shift + int(offs[t]):shift + int(offs[t + 1])] for t in range(len(numel))]


def empty_like_list(tensors: List[torch.Tensor], fill: float = float("nan")) -> List[torch.Tensor]:
    return [torch.full_like(t, fill) for t in tensors]


def gather_flat(tensors: List[torch.Tensor]) -> np.ndarray:
    if not tensors:
        return np.zeros(0, np.float32)
    return torch.cat([t.reshape(-1) for t in tensors]).cpu().numpy() if len(tensors) > 1 else tensors[0].reshape(-1).cpu().numpy()


def check_payload(algo: str, gpay: np.ndarray, opay: np.ndarray, what: str) -> bool:
    """Header fields equal, scalar within the bar.  Returns True if the scalar bits agree."""
    gh, oh = O.header(gpay), O.header(opay)
    for key in ("magic", "algo", "n", "k", "levels"):
        assert gh[key] == oh[key], f"{what}: header field {key}: gpu {gh[key]} oracle {oh[key]}"
    assert not gpay[36 if algo == "onebit" else 32:O.HDR].any(), f"{what}: header padding not zero"
    gs, os_ = np.float32(gh["scale"]), np.float32(oh["scale"])
    if algo == "onebit":                         # two scalars: the class means
        g2, o2 = np.float32(gh["scale2"]), np.float32(oh["scale2"])
        assert abs(float(g2) - float(o2)) <= 1e-6 * abs(float(o2)), f"{what}: lower mean gpu {g2!r} oracle {o2!r}"
        assert abs(float(gs) - float(os_)) <= 1e-6 * abs(float(os_)), f"{what}: upper mean gpu {gs!r} oracle {os_!r}"
        return gs.view(np.uint32) == os_.view(np.uint32) and g2.view(np.uint32) == o2.view(np.uint32)
    if algo == "terngrad":
        assert gs == os_, f"{what}: max|p| must be exact: gpu {gs!r} oracle {os_!r}"
    else:
        assert abs(float(gs) - float(os_)) <= 1e-6 * abs(float(os_)), f"{what}: scalar gpu {gs!r} oracle {os_!r}"
    return gs.view(np.uint32) == os_.view(np.uint32)


def run_parity(numel: Sequence[int], algo: str, y: int, W: int, iters: int,
               grads_fn: Callable[[int, int], np.ndarray], *, policy: int = B.MC_PART_EVEN_ELEMS,
               user_bounds: Optional[Sequence[int]] = None, oracle_workers: Optional[Sequence[int]] = None,
               layout: str = "separate", alpha: float = 1.0, check_decompress: bool = True,
               prelude_fn: Optional[Callable[[int], np.ndarray]] = None,
               worker_id: Callable[[int], int] = lambda w: w, iter0: int = 0, **cfgkw) -> Stats:
    """Full protocol on one (tensor list, algorithm, y): compress every (iteration, group, worker) on the GPU,
    compare payload and residual with the oracle for `oracle_workers` (default: all), then decompress-and-sum
    the oracle's payloads on the GPU and compare with the oracle's aggregate.
    prelude_fn(w): gradients that the same context first compresses and decodes into throw-away buffers (nothing of
    it is compared; what it leaves in the context must not disturb the calls that follow)."""
    stats = Stats()
    numel = [int(x) for x in numel]
    aid = ALGOS[algo]
    bounds = B.mc_partition(numel, y, policy, user_bounds)
    assert bounds == list(O.partition(numel, y, policy, user_bounds)), "mc_partition differs from the oracle"
    if algo == "signsgd":
        cfgkw.setdefault("use_ef", 0)
    ctx = B.Context(aid, numel, bounds, **cfgkw)
    ocfg = O.Config(aid, **cfgkw)
    ef = ocfg.use_ef != 0
    offs = np.concatenate([[0], np.cumsum(numel)]).astype(np.int64)
    goff = [int(offs[bounds[j]]) for j in range(y)]
    gn = [int(offs[bounds[j + 1]] - offs[bounds[j]]) for j in range(y)]
    workers = list(range(W))
    owork = workers if oracle_workers is None else list(oracle_workers)
    for j in range(y):
        assert ctx.group_numel(j) == gn[j]
        assert ctx.payload_bytes(j) == O.payload_bytes(ocfg, gn[j])
        pad = (-gn[j]) % 32 if algo == "dgc" else 0          # DGC's second vector starts on a 128-byte line
        assert ctx.state_bytes(j) == O.HDR + 4 * (O.state_floats(ocfg, gn[j]) + pad)
        assert ctx.group_k(j) == (O.sparse_capacity(ocfg, gn[j]) if algo in ("topk", "dgc", "randk") else 0)

    gstate = [[torch.zeros(ctx.state_bytes(j), dtype=torch.uint8, device=DEV) if ef else None for j in range(y)] for _ in workers]
    gpay = [[torch.full((ctx.payload_bytes(j),), 0xAB, dtype=torch.uint8, device=DEV) for j in range(y)] for _ in workers]
    ostate: Dict[int, List[np.ndarray]] = {w: [O.new_state(ocfg, gn[j]) if ef else None for j in range(y)] for w in owork}
    opay: Dict[int, List[Optional[np.ndarray]]] = {w: [None] * y for w in owork}

    if prelude_fn is not None:
        for j in range(y):
            pays = []
            for w in workers:
                d = device_tensors(prelude_fn(w), numel, layout)
                st = torch.zeros(ctx.state_bytes(j), dtype=torch.uint8, device=DEV) if ef else None
                pays.append(torch.zeros(ctx.payload_bytes(j), dtype=torch.uint8, device=DEV))
                ctx.mc_compress(j, w, 1 << 20, d[bounds[j]:bounds[j + 1]], st, pays[-1])
            sink = empty_like_list(device_tensors(np.zeros(int(offs[-1]), np.float32), numel, layout))
            ctx.mc_decompress_sum(j, pays, alpha, sink[bounds[j]:bounds[j + 1]])
            assert ctx.mc_last_device_status() == B.MC_OK

    for it in range(iters):
        flats = {w: grads_fn(w, it) for w in workers}
        dev = {w: device_tensors(flats[w], numel, layout) for w in workers}
        for j in range(y):
            for w in workers:
                ctx.mc_compress(j, worker_id(w), iter0 + it, dev[w][bounds[j]:bounds[j + 1]], gstate[w][j], gpay[w][j])
        torch.cuda.synchronize()
        for j in range(y):
            for w in owork:
                what = f"{algo} y={y} it={it} group={j} worker={w}"
                g = flats[w][goff[j]:goff[j] + gn[j]]
                before = None if not ef else ostate[w][j].copy()
                op, _ = O.compress(ocfg, g, ostate[w][j], group_off=goff[j], worker=worker_id(w), it=iter0 + it)
                gp = gpay[w][j].cpu().numpy()
                if not check_payload(algo, gp, op, what):
                    stats.conditional += 1
                    stats.notes.append(f"{what}: scalar differs within 1e-6, oracle re-encoded with the GPU scalar")
                    if ef:
                        ostate[w][j][:] = before
                    gh = O.header(gp)
                    op, _ = O.compress(ocfg, g, ostate[w][j], group_off=goff[j], worker=worker_id(w), it=iter0 + it,
                                       scale_in=(gh["scale"], gh["scale2"]) if algo == "onebit" else gh["scale"])
                assert gp.size == op.size
                if not np.array_equal(gp, op):
                    bad = np.nonzero(gp != op)[0]
                    raise AssertionError(f"{what}: payload differs at {bad.size} bytes, first at byte {bad[0]} "
                                         f"(gpu {gp[bad[0]]:#x} oracle {op[bad[0]]:#x})")
                if ef:
                    e = torch.empty(O.state_floats(ocfg, gn[j]), dtype=torch.float32, device=DEV)
                    ctx.mc_state_export_residual(j, gstate[w][j], e)
                    ge = e.cpu().numpy()
                    if not same_bits(ge, ostate[w][j]):
                        bad = np.nonzero(u32(ge) != u32(ostate[w][j]))[0]
                        raise AssertionError(f"{what}: residual differs at {bad.size} elements, first {bad[0]}: "
                                             f"gpu {ge[bad[0]]!r} oracle {ostate[w][j][bad[0]]!r}")
                opay[w][j] = op
                stats.compress_checks += 1

    if check_decompress and len(owork) == W:
        outs = empty_like_list(device_tensors(np.zeros(int(offs[-1]), np.float32), numel, layout))
        for j in range(y):
            up = [torch.from_numpy(opay[w][j]).to(DEV) for w in workers]
            ctx.mc_decompress_sum(j, up, alpha, outs[bounds[j]:bounds[j + 1]])
            assert ctx.mc_last_device_status() == B.MC_OK
            got = gather_flat(outs[bounds[j]:bounds[j + 1]])
            want = O.decompress_sum([opay[w][j] for w in workers], gn[j], alpha)
            if not same_bits(got, want):
                bad = np.nonzero(u32(got) != u32(want))[0]
                raise AssertionError(f"{algo} y={y} group={j}: aggregate differs at {bad.size} elements, first {bad[0]}: "
                                     f"gpu {got[bad[0]]!r} oracle {want[bad[0]]!r}")
            stats.decompress_checks += 1
    ctx.close()
    return stats


def workload_grads(wl: WL.Workload, shared_fraction: float = 0.0, cache: Optional[dict] = None):
    def fn(w: int, it: int) -> np.ndarray:
        key = (wl.cfg, w, it, shared_fraction)
        if cache is not None and key in cache:
            return cache[key]
        x = WL.gradients_flat(wl, w, it, shared_fraction)
        if cache is not None:
            cache[key] = x
        return x
    return fn
