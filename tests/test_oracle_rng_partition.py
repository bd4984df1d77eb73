"""Pins for the oracle's random numbers, partition policies and workload shapes.

Everything here runs on the CPU.  Each check ties the oracle to something other
than itself: published known-answer vectors, combinatorial counts from the
paper's Lemma 1, closed forms, or properties that hold by definition.
"""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import oracle as O
from paper_2103_15195_amd import workloads as WL


def _facts(golden_dir):
    out = {}
    for line in open(os.path.join(golden_dir, "paper_facts.txt")):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = int(line[1])
    return out


# ---------------------------------------------------------------- Philox ----
def test_philox_known_answers(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        got = O.philox4x32_10(v[0:4], v[4:6])
        assert [int(x) for x in got] == v[6:10]


def test_uniform_range_mean_and_keying():
    u = np.array([O.uniform(7, 1, 2, i) for i in range(20000)], dtype=np.float64)
    assert u.min() >= 0.0 and u.max() < 1.0
    # mean 1/2, variance 1/12: 5 sigma of the sample mean
    assert abs(u.mean() - 0.5) < 5 * math.sqrt(1 / 12 / u.size)
    assert abs(u.var() - 1 / 12) < 0.005
    # multiples of 2^-24 (24 random bits, exact in fp32)
    assert np.all(u * 2 ** 24 == np.floor(u * 2 ** 24))
    # four consecutive elements share one Philox block: counter = index // 4, lane = index % 4
    blk = O.philox4x32_10([5, 0, 1, 2], [7, 0])
    for lane in range(4):
        assert O.uniform(7, 1, 2, 20 + lane) == float(blk[lane] >> 8) * 2.0 ** -24
    # high words of index, iteration and seed reach the counter / key
    big = (3 << 34) + 1
    blk = O.philox4x32_10([(big >> 2) & 0xFFFFFFFF, big >> 34, 9, 4], [0x89ABCDEF, 0x01234567])
    assert O.uniform(0x0123456789ABCDEF, 9, 4, big) == float(blk[1] >> 8) * 2.0 ** -24
    # distinct worker / iteration / seed give distinct streams
    base = [O.uniform(7, 1, 2, i) for i in range(64)]
    for other in ([O.uniform(8, 1, 2, i) for i in range(64)], [O.uniform(7, 2, 2, i) for i in range(64)],
                  [O.uniform(7, 1, 3, i) for i in range(64)]):
        assert sum(a == b for a, b in zip(base, other)) < 4


# ------------------------------------------------------------- partition ----
def _all_contiguous_partitions(N, y):
    for cuts in itertools.combinations(range(1, N), y - 1):
        yield (0,) + cuts + (N,)


def test_lemma1_partition_counts():
    # Lemma 1: C(N-1, y-1) contiguous partitions into y groups, 2^(N-1) in total;
    # every one of them is accepted unchanged by the USER policy
    for N in range(1, 10):
        numel = list(range(1, N + 1))
        total = 0
        for y in range(1, N + 1):
            parts = list(_all_contiguous_partitions(N, y))
            assert len(parts) == math.comb(N - 1, y - 1)
            total += len(parts)
            for b in parts:
                assert tuple(O.partition(numel, y, O.PART_USER, b)) == b
        assert total == 2 ** (N - 1)


@pytest.mark.parametrize("N,y", [(161, 2), (161, 3), (314, 4), (7, 7), (10, 3), (5, 1)])
def test_even_count_policy(N, y):
    b = O.partition([1] * N, y, O.PART_EVEN_COUNT)
    sizes = np.diff(b)
    assert b[0] == 0 and b[-1] == N and sizes.sum() == N
    assert sizes.max() - sizes.min() <= 1 and sizes.min() >= 1
    if (N, y) == (161, 2):
        assert list(b) == [0, 80, 161]


def test_even_elems_policy_bruteforce():
    rng = np.random.default_rng(3)
    for trial in range(60):
        N = int(rng.integers(1, 10))
        numel = rng.integers(0, 50, size=N).tolist() if trial % 3 else rng.integers(1, 1000, size=N).tolist()
        D = sum(numel)
        prefix = np.concatenate([[0], np.cumsum(numel)])
        for y in range(1, N + 1):
            b = O.partition(numel, y, O.PART_EVEN_ELEMS)
            assert b[0] == 0 and b[-1] == N and np.all(np.diff(b) >= 1)
            assert tuple(b) in set(_all_contiguous_partitions(N, y))
            for j in range(1, y):
                lo, hi = b[j - 1] + 1, N - (y - j)
                # the unclamped boundary: first t whose prefix reaches the j/y share of D
                want = next(t for t in range(N + 1) if prefix[t] * y >= j * D)
                assert b[j] == min(max(want, lo), hi)


def test_even_elems_balances_real_model():
    wl = WL.workload(2)
    numel = wl.numel
    for y in (2, 3, 4):
        b = O.partition(numel, y, O.PART_EVEN_ELEMS)
        sizes = np.array([numel[b[j]:b[j + 1]].sum() for j in range(y)])
        assert sizes.sum() == wl.total
        # no group may exceed its even share by more than the largest tensor
        assert sizes.max() <= wl.total / y + numel.max()


def test_partition_errors():
    with pytest.raises(ValueError):
        O.partition([1, 2, 3], 4, O.PART_EVEN_COUNT)      # y > N
    with pytest.raises(ValueError):
        O.partition([1, 2, 3], 0, O.PART_EVEN_COUNT)      # y < 1
    with pytest.raises(ValueError):
        O.partition([1, 2, 3], 2, O.PART_USER, [0, 0, 3])  # empty group
    with pytest.raises(ValueError):
        O.partition([1, 2, 3], 2, O.PART_USER, [0, 2, 2])  # does not end at N


# -------------------------------------------------------------- workloads ---
def test_workload_shapes_match_paper(golden_dir):
    f = _facts(golden_dir)
    assert len(WL.workload(2).shapes) == f["resnet50_tensors"]
    assert len(WL.workload(3).shapes) == f["resnet101_tensors"]
    # parameter counts of the standard architectures
    assert WL.workload(0).total == 784 * 256 + 256 + 256 * 256 + 256 + 2560 + 10
    assert WL.workload(2).total == 25_557_032
    assert WL.workload(3).total == 44_549_160
    assert (len(WL.workload(1).shapes), WL.workload(1).total) == (65, 272_474)
    assert (len(WL.workload(4).shapes), WL.workload(4).total) == (201, 44_454_513)


def test_workload_values_seeded():
    wl = WL.workload(1)
    a = WL.gradients(wl, 0, 0)
    b = WL.gradients(wl, 0, 0)
    c = WL.gradients(wl, 1, 0)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    assert not np.array_equal(a[0], c[0])
    assert all(x.dtype == np.float32 and x.size == n for x, n in zip(a, wl.numel))
    std = WL.tensor_std(wl)
    assert std.min() >= 1e-4 and std.max() <= 1e-1
    big = int(np.argmax(wl.numel))
    assert abs(a[big].std() / std[big] - 1) < 0.05


def test_payload_sizes_follow_paper_settings(golden_dir):
    f = _facts(golden_dir)
    n = WL.workload(2).total
    ppm = (100 - f["sparsity_percent"]) * 10000
    assert O.topk_count(n, ppm) == n // 100
    assert O.payload_bytes(O.Config(O.QSGD, qsgd_bits=f["qsgd_bits_per_element"]), n) == O.HDR + n  # 8 bits / element
    assert O.payload_bytes(O.Config(O.EFSIGN), n) == O.HDR + 4 * ((n + 31) // 32)                 # 1 bit / element
    # 99 % sparsity: an index and a value per kept entry, and the directory of the index list (one entry per 4096 elements and one more)
    assert O.payload_bytes(O.Config(O.TOPK, ratio_ppm=ppm), n) == O.HDR + 8 * (n // 100) + 4 * ((n + 4095) // 4096 + 1)
    assert O.topk_count(50, 10000) == 1 and O.topk_count(0, 10000) == 0 and O.topk_count(3, 10 ** 6) == 3
