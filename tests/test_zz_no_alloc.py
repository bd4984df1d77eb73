"""The allocation-free entry point, mc_compress_static, against mc_compress through the C ABI: same payload and
state, bit for bit, on two calls in a row of which the second has the smaller input (the static scratch array
keeps what the first call left in it)."""
import numpy as np
import pytest
import torch

from paper_2103_15195_amd import binding as B

import harness as H

pytestmark = pytest.mark.gpu

DENSE = ["efsign", "onebit", "qsgd", "terngrad", "fp16", "signum", "signsgd"]


def _run(ctx, entry, group, grads, it):
    state = torch.zeros(ctx.state_bytes(group), dtype=torch.uint8, device=H.DEV)
    pay = torch.full((ctx.payload_bytes(group),), 0xCD, dtype=torch.uint8, device=H.DEV)
    outs = []
    for i in range(2):                      # two iterations: the second one reads the state the first one left
        entry(group, 3, it + i, grads, None if ctx.algo == B.MC_ALGO_SIGNSGD else state, pay)
        torch.cuda.synchronize()
        outs.append((pay.cpu().numpy().copy(), state.cpu().numpy().copy()))
    return outs


@pytest.mark.parametrize("algo", DENSE)
def test_static_entry_equals_mc_compress_twice_in_a_row(algo):
    # group 0: 41 tensors, 5 tiles and a ragged tail; group 1: much smaller (its tiles reuse the first partials)
    rng = np.random.default_rng(11)
    big = [int(x) for x in rng.integers(1, 1200, size=40)] + [3 * 4096 + 77]
    small = [700, 13, 2048 + 5]
    numel = big + small
    bounds = [0, len(big), len(numel)]
    flat = rng.standard_normal(sum(numel), dtype=np.float32) * np.float32(0.02)
    dev = H.device_tensors(flat, numel)
    ctx = B.Context(algo, numel, bounds, seed=5)
    ref = B.Context(algo, numel, bounds, seed=5)
    for group in (0, 1):                    # the larger group first, then the smaller one
        g = dev[bounds[group]:bounds[group + 1]]
        got = _run(ctx, ctx.mc_compress_static, group, g, 7)
        want = _run(ref, ref.mc_compress, group, g, 7)
        for (gp, gs), (wp, ws) in zip(got, want):
            assert np.array_equal(gp, wp), f"{algo} group {group}: payload differs from mc_compress"
            assert np.array_equal(gs, ws), f"{algo} group {group}: state differs from mc_compress"
    ctx.close(); ref.close()


def test_static_entry_limits():
    L = B.lib()
    assert L.mc_static_scratch_bytes() == 3 * 8 * (L.mc_static_max_elems() // 4096)
    n = 5000
    g = torch.randn(n, device=H.DEV)
    sp = B.Context("topk", [n], [0, 1])
    st = torch.zeros(sp.state_bytes(0), dtype=torch.uint8, device=H.DEV)
    pay = torch.zeros(sp.payload_bytes(0), dtype=torch.uint8, device=H.DEV)
    with pytest.raises(B.McError) as e:
        sp.mc_compress_static(0, 0, 0, [g], st, pay)           # a sparsifier: not served
    assert e.value.status == B.MC_ERR_INVALID_ARG
    sp.close()
    # one element above the limit: rejected before anything is launched (the buffers passed are far too small on purpose)
    big = B.Context("efsign", [L.mc_static_max_elems() + 1], [0, 1])
    with pytest.raises(B.McError) as e:
        big.mc_compress_static(0, 0, 0, [g], st, pay)
    assert e.value.status == B.MC_ERR_RANGE
    big.close()
