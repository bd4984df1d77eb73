"""A merged group close to the largest the library accepts (2^32 - 2^24 elements; flat indices are 32-bit), through
the C ABI: 4 259 840 000 elements, more than 2^31, in ragged tensors whose boundaries lie beyond element 2^31.

The oracle cannot run on 17 GB in reasonable time, so the gradient is periodic: a seeded base vector of L elements
repeated 4096 times (L is a multiple of 64 and of 1000, not of 1024, so periods are ragged against chunks and tiles).
What the method computes on it follows from what the oracle computes on one period:
  * EF-Sign, OneBit, SigNUM, FP16: elementwise once the group scalar is known, and the scalar (a mean) is that of
    one period.  Every period of the payload body and of the residual must equal the oracle's on the base.
  * Top-k, DGC: every key occurs 4096 times, so the k = 4096 k_L largest are the copies of the k_L largest of
    the base (the test checks that rank k_L and k_L + 1 of the base differ): indices idx_L + r L for all r, ascending.
  * QSGD, TernGrad draw one random number per element from its group-wide index, so periods differ: the oracle
    runs on sampled periods with group_off = r L (the periods around element 2^31 among them).  TernGrad's scalar is
    the maximum (that of the base, exact); QSGD's norm is 64 times the base's (4096 = 64^2), compared within 1e-6.
    From the second iteration on their residuals differ from period to period too, and so does the scalar's
    share of every period: it is then checked against an fp64 reduction (torch, on the device) of g + e with e
    the residual the library exports -- a consistency check; the residual itself is compared on the sampled periods.
In every case the oracle's encode step takes the GPU's scalar as input once that scalar has passed its own check
(the same protocol as the other parity tests), so payload bytes and residuals are compared bit for bit.
Then two workers' payloads are decompressed-and-summed at full size and compared period by period.
"""
import gc

import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2103_15195_amd import binding as B

import harness as H

pytestmark = pytest.mark.gpu

L = 1_040_000
REPS = 4096
N = L * REPS
CAP = (1 << 32) - (1 << 24)
NUMEL = [(1 << 31) + 777, 5, 0, 3, 1_000_003, 1]
NUMEL.append(N - sum(NUMEL))
OFFS = np.concatenate([[0], np.cumsum(NUMEL)]).astype(np.int64)
# periods compared for the schemes that draw random numbers: the ends, and those around element 2^31
SAMPLE = [0, 1, 2063, 2064, 2065, 4095]
PLANES = ("efsign", "onebit", "signum")
RANDOM = ("qsgd", "terngrad")


def base_vector(worker, it):
    rng = np.random.default_rng([2103, worker, it])
    return (rng.standard_normal(L) * np.exp(rng.standard_normal(L)) * 0.01).astype(np.float32)


def views(flat):
    return [flat[int(OFFS[t]):int(OFFS[t + 1])] for t in range(len(NUMEL))]


def on_device(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(H.DEV)


def periods_equal(buf, want):
    """Every period of a device buffer equals `want` (one period, numpy), compared as bytes."""
    w = on_device(want.view(np.uint8))
    return bool((buf.view(REPS, w.numel()) == w[None, :]).all())


def period_of(buf, r, nbytes):
    return buf[r * nbytes:(r + 1) * nbytes].cpu().numpy()


def gpu_scalars(algo, hdr):
    if algo == "onebit":
        return (hdr["scale"], hdr["scale2"])
    return hdr["scale"] if algo in ("efsign", "qsgd", "terngrad") else None


def check_scalar(algo, hdr, ocfg, base, ostate, worker, it):
    """The GPU's group scalar against what the oracle computes on one period (on a copy of its state)."""
    if gpu_scalars(algo, hdr) is None:
        return
    trial = None if ostate is None else ostate.copy()
    opay, _ = O.compress(ocfg, base, trial, worker=worker, it=it)
    oh = O.header(opay)
    if algo == "terngrad":
        assert np.float32(hdr["scale"]) == np.float32(oh["scale"]), "max |p| must be exact"
        return
    pairs = [(hdr["scale"], oh["scale"] * (64.0 if algo == "qsgd" else 1.0))]      # ||p|| over 4096 periods = 64 ||base||
    if algo == "onebit":
        pairs.append((hdr["scale2"], oh["scale2"]))
    for got, want in pairs:
        assert abs(got - want) <= 1e-6 * abs(want), f"{algo}: group scalar gpu {got!r}, from the oracle {want!r}"


def check_scalar_by_reduction(algo, hdr, ctx, st, flat):
    """QSGD / TernGrad after the first iteration: the scalar of p = g + e over the whole group, e exported by the library."""
    e = torch.empty(N, dtype=torch.float32, device=H.DEV)
    ctx.mc_state_export_residual(0, st, e)
    sq, mx = 0.0, 0.0
    for a in range(0, N, 1 << 28):
        pchunk = flat[a:a + (1 << 28)] + e[a:a + (1 << 28)]
        if algo == "qsgd":
            sq += float((pchunk.double() ** 2).sum())
        else:
            mx = max(mx, float(pchunk.abs().max()))
    del e
    if algo == "qsgd":
        want = float(np.sqrt(sq))
        assert abs(hdr["scale"] - want) <= 1e-6 * want, f"qsgd: norm gpu {hdr['scale']!r}, fp64 reduction {want!r}"
    else:
        assert np.float32(hdr["scale"]) == np.float32(mx), f"terngrad: max gpu {hdr['scale']!r}, reduction {mx!r}"


def body_period_bytes(algo, k_l):
    return {"efsign": L // 8, "onebit": L // 8, "signum": L // 8, "fp16": 2 * L, "qsgd": L}.get(algo)


def check_payload(algo, pay, hdr, opay_of, k_l):
    """pay: the GPU payload (device bytes); opay_of[r]: the oracle's payload of period r (r = 0 stands for all
    periods when the scheme draws no random numbers)."""
    assert hdr["magic"] == 0x3150434D and hdr["algo"] == H.ALGOS[algo] and hdr["n"] == N
    body = pay[O.HDR:]
    if algo in ("topk", "dgc"):
        assert hdr["k"] == REPS * k_l
        k = hdr["k"]
        idx_l, val_l = O.sparse_view(opay_of[0])
        assert idx_l.size == k_l
        got_idx = body[:4 * k].view(torch.int32).to(torch.int64) & 0xFFFFFFFF
        want_idx = (on_device(idx_l.astype(np.int64))[None, :] + (torch.arange(REPS, device=H.DEV, dtype=torch.int64) * L)[:, None])
        assert torch.equal(got_idx.view(REPS, k_l), want_idx), f"{algo}: indices differ"
        assert periods_equal(body[4 * k:8 * k], val_l), f"{algo}: values differ"
        # the directory that ends the payload: entries of the (ascending) index list below each multiple of 4096
        spans = (N + 4095) // 4096
        got_dir = body[8 * k:8 * k + 4 * (spans + 1)].view(torch.int32).to(torch.int64) & 0xFFFFFFFF
        want_dir = torch.searchsorted(got_idx.contiguous(), torch.arange(spans + 1, device=H.DEV, dtype=torch.int64) * 4096)
        assert torch.equal(got_dir, want_dir), f"{algo}: directory differs"
        return
    if algo == "terngrad":
        nb, lb = N // 8, L // 8
        for r, opay in opay_of.items():
            want = opay[O.HDR:]
            assert np.array_equal(period_of(body[:nb], r, lb), want[:lb]), f"terngrad: non-zero plane of period {r} differs"
            assert np.array_equal(period_of(body[nb:2 * nb], r, lb), want[lb:2 * lb]), f"terngrad: sign plane of period {r} differs"
        return
    lb = body_period_bytes(algo, k_l)
    if algo in RANDOM:
        for r, opay in opay_of.items():
            assert np.array_equal(period_of(body, r, lb), opay[O.HDR:O.HDR + lb]), f"{algo}: codes of period {r} differ"
    else:
        assert periods_equal(body[:REPS * lb], opay_of[0][O.HDR:O.HDR + lb]), f"{algo}: payload body differs"


def check_residual(algo, ctx, st, ostate_of):
    if algo == "dgc":
        e = torch.empty(2 * N, dtype=torch.float32, device=H.DEV)
    else:
        e = torch.empty(N, dtype=torch.float32, device=H.DEV)
    ctx.mc_state_export_residual(0, st, e)
    torch.cuda.synchronize()
    if algo in RANDOM:
        for r, ost in ostate_of.items():
            assert H.same_bits(e[r * L:(r + 1) * L].cpu().numpy(), ost), f"{algo}: residual of period {r} differs"
    elif algo == "dgc":
        ost = ostate_of[0]
        assert periods_equal(e[:N].view(torch.uint8), ost[:L]), "dgc: accumulated gradient v differs"
        assert periods_equal(e[N:].view(torch.uint8), ost[L:]), "dgc: momentum u differs"
    else:
        assert periods_equal(e.view(torch.uint8), ostate_of[0]), f"{algo}: residual differs"
    del e


def run_worker(algo, ctx, ocfg, worker, iters, k_l):
    """Compress `iters` iterations of one worker at full size, each checked against the oracle.  Returns the GPU
    payload of the last iteration and the oracle's period payloads of it."""
    periods = SAMPLE if algo in RANDOM else [0]
    stateful = O.state_floats(ocfg, L) > 0
    st = torch.zeros(ctx.state_bytes(0), dtype=torch.uint8, device=H.DEV) if stateful else None
    pay = torch.zeros(ctx.payload_bytes(0), dtype=torch.uint8, device=H.DEV)
    ostate_of = {r: (O.new_state(ocfg, L) if stateful else None) for r in periods}
    opay_of = {}
    for it in range(iters):
        base = base_vector(worker, it)
        if algo in ("topk", "dgc"):          # the selection is periodic only if the base has no tie across rank k_L
            trial = ostate_of[0].copy()
            ppay, _ = O.compress(ocfg, base, trial, worker=worker, it=it)
            _, pval = O.sparse_view(ppay)
            # the oracle's state after the call holds p with the kept entries removed: its largest is rank k_L + 1
            rest = np.abs(trial[:L]).max()
            assert np.abs(pval).min() > rest, "base vector has a tie at the threshold: choose another seed"
        flat = on_device(base).repeat(REPS)
        before = st.clone() if algo in RANDOM and it > 0 else None
        ctx.mc_compress(0, worker, it, views(flat), st, pay)
        torch.cuda.synchronize()
        assert ctx.mc_last_device_status() == B.MC_OK
        hdr = O.header(pay[:O.HDR].cpu().numpy())
        # the scalar first, then the oracle's encode with the GPU's scalar
        if before is not None:
            check_scalar_by_reduction(algo, hdr, ctx, before, flat)
        else:
            check_scalar(algo, hdr, ocfg, base, ostate_of[periods[0]], worker, it)
        del flat, before
        for r in periods:
            opay_of[r], _ = O.compress(ocfg, base, ostate_of[r], group_off=r * L, worker=worker, it=it,
                                       scale_in=gpu_scalars(algo, hdr))
        check_payload(algo, pay, hdr, opay_of, k_l)
        if stateful:
            check_residual(algo, ctx, st, ostate_of)
        print(f"[max size {algo}] worker {worker} iteration {it}: payload and state agree", flush=True)
    return pay, opay_of


def run_maxsize(algo, ppm=10000, iters=2, **kw):
    gc.collect()
    torch.cuda.empty_cache()
    ctx = B.Context(algo, NUMEL, [0, len(NUMEL)], ratio_ppm=ppm, seed=77, **kw)
    ocfg = O.Config(H.ALGOS[algo], ratio_ppm=ppm, seed=77, **kw)
    assert ctx.group_numel(0) == N
    k_l = O.topk_count(L, ppm) if algo in ("topk", "dgc") else 0
    if k_l:
        assert ctx.group_k(0) == REPS * k_l == O.topk_count(N, ppm)
    pay0, opay0 = run_worker(algo, ctx, ocfg, 0, iters, k_l)
    pay1, opay1 = run_worker(algo, ctx, ocfg, 1, 1, k_l)
    # decompress-and-sum of the two payloads into ragged tensors, compared period by period
    out = torch.full((N,), float("nan"), dtype=torch.float32, device=H.DEV)
    ctx.mc_decompress_sum(0, [pay0, pay1], 0.5, views(out))
    torch.cuda.synchronize()
    assert ctx.mc_last_device_status() == B.MC_OK
    if algo in RANDOM:
        for r in SAMPLE:
            want = O.decompress_sum([opay0[r], opay1[r]], L, 0.5)
            assert H.same_bits(out[r * L:(r + 1) * L].cpu().numpy(), want), f"{algo}: sum of period {r} differs"
    else:
        want = O.decompress_sum([opay0[0], opay1[0]], L, 0.5)
        assert periods_equal(out.view(torch.uint8), want), f"{algo}: aggregated sum differs"
    print(f"[max size {algo}] decompress-and-sum of 2 workers agrees", flush=True)
    ctx.close()
    del out, pay0, pay1
    gc.collect()
    torch.cuda.empty_cache()


def test_group_size_limit():
    """One element below the limit is accepted, the limit itself is refused with MC_ERR_RANGE (no kernel runs)."""
    ctx = B.Context("efsign", [CAP - 1], [0, 1])
    assert ctx.group_numel(0) == CAP - 1
    ctx.close()
    ctx = B.Context("efsign", [CAP - 7, 0, 6], [0, 3])
    assert ctx.group_numel(0) == CAP - 1
    ctx.close()
    for numel, bounds in (([CAP], [0, 1]), ([CAP - 7, 7], [0, 2]), ([5, CAP - 7, 7], [0, 1, 3])):
        with pytest.raises(B.McError) as err:
            B.Context("efsign", numel, bounds)
        assert err.value.status == B.MC_ERR_RANGE
    ctx = B.Context("efsign", [CAP - 7, 7], [0, 1, 2])         # the limit is per group
    ctx.close()


@pytest.mark.parametrize("algo", ["efsign", "onebit", "signum", "fp16", "qsgd", "terngrad"])
def test_maxsize_dense(algo):
    run_maxsize(algo)


@pytest.mark.parametrize("algo,ppm", [("topk", 10000), ("dgc", 1000)])
def test_maxsize_sparse(algo, ppm):
    run_maxsize(algo, ppm=ppm)
