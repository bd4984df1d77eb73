"""CPU-side checks of the C-ABI library: it loads, exports every symbol the public
header declares, and its host-only logic (partition policies, argument validation)
agrees with the oracle.  No kernel is launched here."""
import ctypes as C
import itertools
import os
import re

import numpy as np
import pytest

from oracle import oracle as O
from paper_2103_15195_amd import binding as B
from paper_2103_15195_amd import workloads as WL

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "mergecomp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mc_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    syms = declared_symbols()
    assert {"mc_partition", "mc_compress", "mc_decompress_sum"} <= set(syms)
    L = B.lib()
    for s in syms:
        assert hasattr(L, s), f"{s} declared in include/mergecomp.h but not exported"
    assert sorted(B.EXPORTS) == syms
    assert B.lib().mc_version().decode().startswith("mergecomp")


def test_partition_matches_oracle_on_models():
    for cfg in range(5):
        wl = WL.workload(cfg)
        numel = wl.numel.tolist()
        for y in set(wl.ys) | {1, 2, 3, len(numel)}:
            for pol in (B.MC_PART_EVEN_COUNT, B.MC_PART_EVEN_ELEMS):
                assert B.mc_partition(numel, y, pol) == list(O.partition(numel, y, pol))


def test_partition_matches_oracle_bruteforce():
    rng = np.random.default_rng(5)
    for trial in range(200):
        N = int(rng.integers(1, 9))
        numel = rng.integers(0, 40, size=N).tolist()
        for y in range(1, N + 1):
            for pol in (B.MC_PART_EVEN_COUNT, B.MC_PART_EVEN_ELEMS):
                assert B.mc_partition(numel, y, pol) == list(O.partition(numel, y, pol)), (numel, y, pol)
            for cuts in itertools.combinations(range(1, N), y - 1):
                b = [0, *cuts, N]
                assert B.mc_partition(numel, y, B.MC_PART_USER, b) == b


def test_partition_error_codes():
    def status(*a, **k):
        with pytest.raises(B.McError) as e:
            B.mc_partition(*a, **k)
        return e.value.status
    assert status([1, 2, 3], 4) == B.MC_ERR_RANGE
    assert status([1, 2, 3], 0) == B.MC_ERR_INVALID_ARG
    assert status([1, -2, 3], 2) == B.MC_ERR_INVALID_ARG
    assert status([1, 2, 3], 2, 7) == B.MC_ERR_INVALID_ARG
    assert status([1, 2, 3], 2, B.MC_PART_USER) == B.MC_ERR_INVALID_ARG
    assert status([1, 2, 3], 2, B.MC_PART_USER, [0, 0, 3]) == B.MC_ERR_RANGE
    assert status([1, 2, 3], 2, B.MC_PART_USER, [0, 2, 2]) == B.MC_ERR_RANGE
    L = B.lib()
    assert L.mc_partition(None, 3, 1, 0, None, None) == B.MC_ERR_INVALID_ARG


def test_ctx_create_rejects_bad_arguments_before_touching_a_device():
    L = B.lib()
    numel = (C.c_int64 * 3)(4, 5, 6)
    bounds = (C.c_int32 * 2)(0, 3)
    h = C.c_void_p()

    def create(cfg, nm=numel, n=3, bd=bounds, y=1):
        return L.mc_ctx_create(C.byref(h), C.byref(cfg), nm, n, bd, y)
    ok = dict(algo=1, use_ef=1, ratio_ppm=10000, qsgd_bits=8, dgc_momentum=0.9, dgc_sample_ppm=0, seed=0)
    for bad in (dict(algo=0), dict(algo=7), dict(use_ef=2), dict(dgc_sample_ppm=1), dict(algo=3, use_ef=0),
                dict(algo=4, qsgd_bits=1), dict(algo=4, qsgd_bits=9), dict(algo=2, ratio_ppm=0),
                dict(algo=2, ratio_ppm=1000001)):
        assert create(B.McConfig(**{**ok, **bad})) == B.MC_ERR_INVALID_ARG, bad
    good = B.McConfig(**ok)
    assert L.mc_ctx_create(None, C.byref(good), numel, 3, bounds, 1) == B.MC_ERR_INVALID_ARG
    assert L.mc_ctx_create(C.byref(h), None, numel, 3, bounds, 1) == B.MC_ERR_INVALID_ARG
    assert create(good, y=4, bd=(C.c_int32 * 5)(0, 1, 2, 3, 3)) == B.MC_ERR_RANGE          # y > N
    assert create(good, bd=(C.c_int32 * 2)(0, 2)) == B.MC_ERR_RANGE                        # does not end at N
    assert create(good, y=2, bd=(C.c_int32 * 3)(0, 0, 3)) == B.MC_ERR_RANGE                # empty group
    assert create(good, nm=(C.c_int64 * 3)(4, -1, 6)) == B.MC_ERR_INVALID_ARG
    assert create(good, nm=(C.c_int64 * 3)(2 ** 31, 2 ** 31, 6)) == B.MC_ERR_RANGE         # group of >= 2^32 - 2^24
    assert h.value is None
    for s in range(-6, 1):
        assert L.mc_strerror(s)
    assert L.mc_payload_bytes(None, 0) == 0 and L.mc_state_bytes(None, 0) == 0 and L.mc_group_numel(None, 0) == -1
    assert L.mc_compress(None, 0, 0, 0, None, None, None, None) == B.MC_ERR_INVALID_ARG
    assert L.mc_decompress_sum(None, 0, None, 1, 1.0, None, None) == B.MC_ERR_INVALID_ARG
