"""The iteration-time model of Section 4.3 and the partition search of Algorithm 2 (CPU only).

Oracle pins: closed forms of the model (one group; a free network gives Lemma 2's y B_h + gamma_h D; a saturated
network), a timeline worked by hand (tests/golden/partition_timeline_example.txt), the single turning point the
proof of Theorem 3 claims for two groups, and the size of the search space (Lemma 1).  The library's routines
(a dynamic programme instead of enumeration) are then compared with the oracle's brute force.
"""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import oracle as O
from paper_2103_15195_amd import binding as B

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "partition_timeline_example.txt")


def model(fwd=0.0, B_h=0.0, gamma_h=0.0, B_g=0.0, gamma_g=0.0):
    return O.TimeModel(fwd, B_h, gamma_h, B_g, gamma_g), B.McTimeModel(fwd, B_h, gamma_h, B_g, gamma_g)


def random_instance(rng, N):
    numel = rng.integers(1, 5000, N)
    numel[rng.integers(0, N)] *= 50                       # one dominant tensor
    bwd = rng.uniform(0.1e-3, 2e-3, N)
    om, bm = model(fwd=float(rng.uniform(0, 5e-3)), B_h=float(rng.uniform(0, 2e-4)), gamma_h=float(rng.uniform(0, 2e-8)),
                   B_g=float(rng.uniform(0, 5e-4)), gamma_g=float(rng.uniform(0, 2e-7)))
    return numel, bwd, om, bm


# ------------------------------------------------------------------ the oracle's model ----
def test_hand_worked_timeline():
    om, bm = model(1.0, 0.1, 0.001, 0.2, 0.002)
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for bounds, F in rows:
        bounds = [int(b) for b in bounds.split(",")]
        assert O.partition_cost([100, 200, 300], [0.5, 0.5, 0.5], om, bounds) == pytest.approx(float(F), rel=1e-12)
        assert B.mc_partition_cost([100, 200, 300], [0.5, 0.5, 0.5], bm, bounds) == pytest.approx(float(F), rel=1e-12)


def test_one_group_has_no_overlap():
    """y = 1: F = A + h(D) + g(D)."""
    rng = np.random.default_rng(0)
    numel, bwd, om, _ = random_instance(rng, 9)
    D, A = int(numel.sum()), om.fwd + bwd.sum()
    want = A + om.B_h + om.gamma_h * D + om.B_g + om.gamma_g * D
    assert O.partition_cost(numel, bwd, om, [0, 9]) == pytest.approx(want, rel=1e-12)


def test_free_network_gives_lemma_2():
    """g = 0: F = A + y B_h + gamma_h D for every partition with y groups (Lemma 2)."""
    rng = np.random.default_rng(1)
    N = 8
    numel, bwd, _, _ = random_instance(rng, N)
    om, _ = model(fwd=0.003, B_h=1e-4, gamma_h=3e-9)
    for y in (1, 2, 3, 5, 8):
        want = 0.003 + bwd.sum() + y * 1e-4 + 3e-9 * numel.sum()
        for cut in itertools.islice(itertools.combinations(range(1, N), y - 1), 12):
            assert O.partition_cost(numel, bwd, om, [0, *cut, N]) == pytest.approx(want, rel=1e-12)


def test_saturated_network_sends_back_to_back():
    """Communication much slower than everything else: after the first group is ready the network never idles,
    F = (forward + back-propagation and compression of group 1) + y B_g + gamma_g D."""
    numel, bwd = [1000, 2000, 3000, 4000], [1e-3] * 4
    om, _ = model(fwd=2e-3, B_h=1e-5, gamma_h=1e-9, B_g=5e-3, gamma_g=1e-5)
    for bounds in ([0, 1, 4], [0, 2, 3, 4], [0, 1, 2, 3, 4]):
        x1 = sum(numel[:bounds[1]])
        first = 2e-3 + sum(bwd[:bounds[1]]) + 1e-5 + 1e-9 * x1
        want = first + (len(bounds) - 1) * 5e-3 + 1e-5 * sum(numel)
        assert O.partition_cost(numel, bwd, om, bounds) == pytest.approx(want, rel=1e-12)


def test_bounds_of_the_model():
    """The GPU is never idle and the network sends everything: F >= A + sum h, F >= ready(1) + sum g, F <= A + sum h + sum g."""
    rng = np.random.default_rng(2)
    for _ in range(50):
        N = int(rng.integers(2, 9))
        numel, bwd, om, _ = random_instance(rng, N)
        y = int(rng.integers(1, N + 1))
        cut = sorted(rng.choice(np.arange(1, N), y - 1, replace=False).tolist())
        F = O.partition_cost(numel, bwd, om, [0, *cut, N])
        A, D = om.fwd + bwd.sum(), numel.sum()
        sh, sg = y * om.B_h + om.gamma_h * D, y * om.B_g + om.gamma_g * D
        assert A + sh - 1e-15 <= F <= A + sh + sg + 1e-15
        assert F >= sg


def test_two_groups_have_a_single_turning_point():
    """Proof of Theorem 3: F({x_1, D - x_1}) falls up to a turning point and rises after it."""
    rng = np.random.default_rng(3)
    for _ in range(20):
        N = 12
        numel = np.full(N, 1000)                          # equal tensors: x_1 grows linearly with the cut
        bwd = np.full(N, 1e-3)
        om, _ = model(fwd=1e-3, B_h=float(rng.uniform(0, 1e-4)), gamma_h=float(rng.uniform(0, 1e-8)),
                      B_g=float(rng.uniform(0, 1e-3)), gamma_g=float(rng.uniform(1e-8, 2e-6)))
        F = [O.partition_cost(numel, bwd, om, [0, c, N]) for c in range(1, N)]
        d = np.sign(np.round(np.diff(F), 15))
        d = d[d != 0]
        assert (np.diff(d) >= 0).all(), F                 # signs go from -1 to +1 at most once


def test_bruteforce_visits_the_whole_search_space():
    """Lemma 1: C(N-1, y-1) partitions with y groups, 2^(N-1) in all; the brute-force minimum is the minimum over them."""
    rng = np.random.default_rng(4)
    N = 7
    numel, bwd, om, _ = random_instance(rng, N)
    total = 0
    for y in range(1, N + 1):
        cuts = list(itertools.combinations(range(1, N), y - 1))
        assert len(cuts) == math.comb(N - 1, y - 1)
        total += len(cuts)
        Fs = [O.partition_cost(numel, bwd, om, [0, *c, N]) for c in cuts]
        bounds, F = O.partition_best(numel, bwd, om, y)
        assert F == min(Fs) and O.partition_cost(numel, bwd, om, bounds) == F
    assert total == 2 ** (N - 1)


def test_algorithm_2_stopping_rules_on_the_oracle():
    numel, bwd = [1000] * 6, [1e-3] * 6
    # free compression, cheap communication start-up: more groups always help a little
    om, _ = model(fwd=1e-3, B_g=1e-5, gamma_g=1e-6)
    Fmin = [O.partition_best(numel, bwd, om, y)[1] for y in range(1, 7)]
    assert all(a > b for a, b in zip(Fmin, Fmin[1:]))
    b, F = O.partition_search(numel, bwd, om, 6, 0.0)                 # alpha = 0: never "too small", runs to Y
    assert len(b) - 1 == 6 and F == Fmin[5]
    b, F = O.partition_search(numel, bwd, om, 3, 0.0)                 # Y caps the search
    assert len(b) - 1 == 3 and F == Fmin[2]
    gains = [(Fmin[y - 2] - Fmin[y - 1]) / Fmin[y - 2] for y in range(2, 7)]
    alpha = (gains[1] + gains[2]) / 2                                 # gains shrink: the first one below alpha is at y = 4
    assert gains[0] > gains[1] > alpha > gains[2]
    b, F = O.partition_search(numel, bwd, om, 6, alpha)
    assert len(b) - 1 == 4 and F == Fmin[3]
    # the gain is measured against F_min(y-1): just above the gain of y = 4 stops there, just below goes on
    assert len(O.partition_search(numel, bwd, om, 6, gains[2] * (1 + 1e-9))[0]) - 1 == 4
    assert len(O.partition_search(numel, bwd, om, 6, gains[2] * (1 - 1e-9))[0]) - 1 > 4
    # expensive per-group start-up: two groups are already worse than one
    om, _ = model(fwd=1e-3, B_h=5e-3, B_g=5e-3, gamma_g=1e-7)
    b, F = O.partition_search(numel, bwd, om, 6, 0.01)
    assert list(b) == [0, 6] and F == O.partition_cost(numel, bwd, om, [0, 6])


# ------------------------------------------------------------- the library against it ----
@pytest.mark.parametrize("seed", range(12))
def test_library_cost_and_search_match_the_bruteforce(seed):
    rng = np.random.default_rng(100 + seed)
    N = int(rng.integers(2, 11))
    numel, bwd, om, bm = random_instance(rng, N)
    for _ in range(5):
        y = int(rng.integers(1, N + 1))
        cut = sorted(rng.choice(np.arange(1, N), y - 1, replace=False).tolist())
        assert B.mc_partition_cost(numel, bwd, bm, [0, *cut, N]) == pytest.approx(O.partition_cost(numel, bwd, om, [0, *cut, N]), rel=1e-12)
    for Y, alpha in [(N, 0.0), (N, 0.02), (max(1, N // 2), 0.001), (1, 0.5), (N + 5, 0.0)]:
        ob, oF = O.partition_search(numel, bwd, om, Y, alpha)
        gb, gF = B.mc_partition_search(numel, bwd, bm, Y, alpha)
        # several partitions may tie: F and the number of groups are unique, the boundaries must attain F
        assert gF == pytest.approx(oF, rel=1e-12) and len(gb) == len(ob)
        assert gb[0] == 0 and gb[-1] == N and all(a < b for a, b in zip(gb, gb[1:]))
        assert O.partition_cost(numel, bwd, om, gb) == pytest.approx(oF, rel=1e-12)


def test_library_inner_minimum_for_every_y():
    """alpha = 0 and a model where more groups always help: the search runs to Y, so F_min(Y) is exposed for each Y."""
    rng = np.random.default_rng(7)
    N = 10
    numel = rng.integers(500, 5000, N)
    bwd = rng.uniform(0.5e-3, 2e-3, N)
    om, bm = model(fwd=1e-3, gamma_h=1e-9, B_g=1e-6, gamma_g=3e-7)
    for Y in range(1, N + 1):
        _, oF = O.partition_best(numel, bwd, om, Y)
        gb, gF = B.mc_partition_search(numel, bwd, bm, Y, 0.0)
        if len(gb) - 1 == Y:
            assert gF == pytest.approx(oF, rel=1e-12)


def test_library_search_on_a_model_sized_list():
    """ResNet-50-sized tensor list (161 tensors): runs in polynomial time and beats or ties both one group and
    the even-by-elements partitions it could have returned."""
    from paper_2103_15195_amd import workloads as WL
    wl = WL.workload(2)
    numel = wl.numel.tolist()
    bwd = [60e-3 * n / wl.total + 20e-6 for n in numel]                      # back-propagation time ~ tensor size
    bm = B.McTimeModel(30e-3, 40e-6, 2.3e-12, 60e-6, 4 * 8 / 100e9 * 0.01)   # 1 % payload over a 100 Gb/s link
    bounds, F = B.mc_partition_search(numel, bwd, bm, 8, 0.002)
    y = len(bounds) - 1
    assert 1 <= y <= 8 and F <= B.mc_partition_cost(numel, bwd, bm, [0, len(numel)]) + 1e-15
    assert F <= B.mc_partition_cost(numel, bwd, bm, B.mc_partition(numel, y)) + 1e-15


@pytest.mark.parametrize("algo,ppm,B_h,gD", [("efsign", 0, 4e-6, 54e-6), ("topk", 10000, 14e-6, 66e-6), ("dgc", 1000, 14e-6, 85e-6)])
def test_search_on_the_benchmarks_timeline_matches_the_bruteforce(algo, ppm, B_h, gD):
    """The inputs the benchmark feeds Algorithm 2 with (the paper's iteration and PCIe figures, an h(x) of the size the GPU
    measures), on the last 24 tensors of the ResNet-50 list, where the oracle can still enumerate every partition."""
    from paper_2103_15195_amd import workloads as WL
    numel = WL.workload(2).numel.tolist()[-24:]
    D = sum(numel)
    bwd, mp = WL.iteration_timeline(numel, B_h, gD / D, WL.sent_bytes_per_elem(algo, ppm))
    assert sum(bwd) == pytest.approx(2.0 / 3.0 * 64e-3) and mp[0] == pytest.approx(64e-3 / 3.0)
    om, bm = O.TimeModel(*mp), B.McTimeModel(*mp)
    for Y, alpha in [(4, 0.01), (4, 0.0), (3, 1e-4)]:
        ob, oF = O.partition_search(numel, bwd, om, Y, alpha)
        gb, gF = B.mc_partition_search(numel, bwd, bm, Y, alpha)
        assert gF == pytest.approx(oF, rel=1e-12) and len(gb) == len(ob)
        assert O.partition_cost(numel, bwd, om, gb) == pytest.approx(oF, rel=1e-12)
        for pol in (B.MC_PART_EVEN_ELEMS, B.MC_PART_EVEN_COUNT):          # what the search returns is no worse than the naive splits
            assert gF <= B.mc_partition_cost(numel, bwd, bm, B.mc_partition(numel, len(gb) - 1, pol)) * (1 + 1e-12)


def test_library_argument_checks():
    _, bm = model(1.0)
    L = B.lib()
    with pytest.raises(B.McError):
        B.mc_partition_cost([1, 2], [0.1, 0.1], bm, [0, 3])
    with pytest.raises(B.McError):
        B.mc_partition_cost([1, 2], [0.1, 0.1], bm, [0, 1, 1, 2])
    with pytest.raises(B.McError):
        B.mc_partition_search([1, 2], [0.1, 0.1], bm, 2, 1.0)
    with pytest.raises(B.McError):
        B.mc_partition_search([1, 2], [0.1, -0.1], bm, 2, 0.1)
    with pytest.raises(B.McError):
        B.mc_partition_search([1, 2], [0.1, 0.1], B.McTimeModel(1.0, -1.0, 0, 0, 0), 2, 0.1)
    assert L.mc_partition_search(None, None, 2, None, 2, 0.1, None, None, None) == B.MC_ERR_INVALID_ARG
