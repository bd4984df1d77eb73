"""Pins for the oracle's DGC with a sampled threshold (CPU only).

The cited DGC work avoids an exact top-k over all values: it takes the threshold that keeps the wanted ratio of a
sample and sends everything that reaches it.  Pinned here by the special case that collapses to the exact selection
(sample = everything), a library sort of the sample, the capacity rule on tied values, conservation of the
accumulators, and the statistics of the kept count.
"""
import numpy as np
import pytest

from oracle import oracle as O


def rand_group(n, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(n) * scale).astype(np.float32)


def keys(x):
    return x.view(np.uint32) & np.uint32(0x7FFFFFFF)


def sample_start(cfg, group_off, worker, it):
    stride = max(1, 1000000 // cfg.dgc_sample_ppm)
    J = group_off >> 2
    r = O.philox4x32_10([J & 0xFFFFFFFF, J >> 32, worker, it & 0xFFFFFFFF], [cfg.seed & 0xFFFFFFFF, cfg.seed >> 32])
    return int(r[group_off & 3]) % stride, stride


def test_sampling_everything_is_the_exact_selection():
    n = 20000
    g = rand_group(n, 1)                                              # distinct magnitudes: no ties at the threshold
    a_cfg = O.Config(O.DGC, ratio_ppm=5000, dgc_momentum=0.5, dgc_sample_ppm=1000000)
    b_cfg = O.Config(O.DGC, ratio_ppm=5000, dgc_momentum=0.5)
    sa, sb = O.new_state(a_cfg, n), O.new_state(b_cfg, n)
    for it in range(3):
        pa, _ = O.compress(a_cfg, g, sa, it=it)
        pb, _ = O.compress(b_cfg, g, sb, it=it)
        ia, va = O.sparse_view(pa)
        ib, vb = O.sparse_view(pb)
        assert O.header(pa)["k"] == O.header(pb)["k"] == 100
        assert np.array_equal(ia, ib) and np.array_equal(va, vb) and np.array_equal(sa, sb)
        assert O.header(pa)["levels"] == 200 and O.header(pb)["levels"] == 0
        dirb = 4 * ((n + 4095) // 4096 + 1)                            # the directory that ends a sparse payload
        assert pa.size == O.HDR + 8 * 200 + dirb and pb.size == O.HDR + 8 * 100 + dirb


@pytest.mark.parametrize("n,ratio,sppm,off,worker,it", [(50000, 10000, 10000, 0, 0, 0), (50000, 10000, 50000, 12345, 3, 9),
                                                        (9999, 100000, 200000, 7, 1, 2), (300, 10000, 10000, 0, 0, 0),
                                                        (300, 800000, 500000, 0, 0, 1)])
def test_threshold_is_the_quantile_of_the_strided_sample(n, ratio, sppm, off, worker, it):
    cfg = O.Config(O.DGC, ratio_ppm=ratio, dgc_momentum=0.0, dgc_sample_ppm=sppm, seed=77)
    g = rand_group(n, n + it)
    st = O.new_state(cfg, n)
    pay, _ = O.compress(cfg, g, st, group_off=off, worker=worker, it=it)
    first, stride = sample_start(cfg, off, worker, it)
    assert stride == 1000000 // sppm
    sample = keys(g)[first::stride]
    cap = min(n, 2 * O.topk_count(n, ratio))
    h = O.header(pay)
    assert h["levels"] == cap == O.sparse_capacity(cfg, n)
    if sample.size:
        ks = max(1, sample.size * ratio // 1000000)
        thr = np.sort(sample)[-ks]
    else:
        thr = 0
    want = np.nonzero(keys(g) >= thr)[0]
    idx, val = O.sparse_view(pay)
    if want.size <= cap:
        assert h["k"] == want.size and np.array_equal(idx, want)
    else:
        assert h["k"] == cap
    assert np.array_equal(val, g[idx]) and (np.diff(idx.astype(np.int64)) > 0).all()
    # unused entries of the payload stay zero
    assert not pay[O.HDR + 4 * h["k"]:O.HDR + 4 * cap].any() and not pay[O.HDR + 4 * cap + 4 * h["k"]:O.HDR + 8 * cap].any()
    # the directory of the index list follows the two lists
    assert np.array_equal(O.sparse_directory(pay), np.searchsorted(idx, np.arange((n + 4095) // 4096 + 1) * 4096, side="left"))
    # momentum 0, zero state: what was sent plus what is remembered is g, exactly; kept entries left both accumulators
    back = st[:n].copy()
    back[idx] += val
    assert np.array_equal(back, g) and not st[:n][idx].any() and not st[n:][idx].any()


def test_sample_offset_moves_with_worker_iteration_and_group():
    cfg = O.Config(O.DGC, dgc_sample_ppm=1000, seed=5)
    starts = {sample_start(cfg, off, w, it)[0] for off in (0, 4096, 99999) for w in range(3) for it in range(3)}
    assert len(starts) > 20 and all(0 <= s < 1000 for s in starts)


def test_capacity_rule_on_tied_values():
    """Above the threshold first, then ties in index order, until the capacity min(n, 2k) is reached."""
    n = 1000
    cfg = O.Config(O.DGC, ratio_ppm=50000, dgc_momentum=0.0, dgc_sample_ppm=1000000)      # k = 50, capacity 100
    g = np.full(n, 0.5, np.float32)
    pay, _ = O.compress(cfg, g, O.new_state(cfg, n))
    idx, _ = O.sparse_view(pay)
    assert O.header(pay)["k"] == 100 and np.array_equal(idx, np.arange(100))
    g[[700, 800, 900]] = [2.0, -3.0, 4.0]                  # three above, everything else tied at the threshold
    pay, _ = O.compress(cfg, g, O.new_state(cfg, n))
    idx, val = O.sparse_view(pay)
    assert O.header(pay)["k"] == 100
    assert np.array_equal(idx, np.concatenate([np.arange(97), [700, 800, 900]]))
    assert list(val[-3:]) == [2.0, -3.0, 4.0]
    # more than the capacity above a threshold taken from an unlucky sample: the first ones in index order
    cfg = O.Config(O.DGC, ratio_ppm=10000, dgc_momentum=0.0, dgc_sample_ppm=100000, seed=1)   # stride 10, k = 10, capacity 20
    first, stride = sample_start(cfg, 0, 0, 0)
    g = np.ones(n, np.float32)
    g[first::stride] = 0.25                                # the sample only sees the small values
    pay, _ = O.compress(cfg, g, O.new_state(cfg, n))
    idx, val = O.sparse_view(pay)
    big = np.nonzero(g == 1.0)[0]
    assert O.header(pay)["k"] == 20 and np.array_equal(idx, big[:20]) and (val == 1.0).all()


def test_kept_count_tracks_k():
    n, ratio = 400000, 10000
    cfg = O.Config(O.DGC, ratio_ppm=ratio, dgc_momentum=0.0, dgc_sample_ppm=50000, seed=9)     # 20000 samples, ks = 200
    k = O.topk_count(n, ratio)
    counts = []
    for it in range(12):
        pay, _ = O.compress(cfg, rand_group(n, 100 + it), O.new_state(cfg, n), it=it)
        counts.append(O.header(pay)["k"])
    counts = np.array(counts)
    # the sample quantile has a relative error of about 1 / sqrt(ks) = 7 %
    assert abs(counts.mean() - k) < 0.1 * k and (counts < 2 * k).all() and counts.std() > 0


def test_payloads_with_a_capacity_decode_and_sum():
    n, W = 5000, 3
    cfg = O.Config(O.DGC, ratio_ppm=20000, dgc_momentum=0.0, dgc_sample_ppm=100000, seed=4)
    pays = [O.compress(cfg, rand_group(n, w), O.new_state(cfg, n), worker=w)[0] for w in range(W)]
    acc = np.zeros(n, np.float32)
    for pay in pays:
        idx, val = O.sparse_view(pay)
        d = np.zeros(n, np.float32)
        d[idx] = val
        assert np.array_equal(O.decode(pay, n), d)
        acc = acc + d
    assert np.array_equal(O.decompress_sum(pays, n, 0.5), np.float32(0.5) * acc)


def test_empty_group_and_momentum_masking():
    cfg = O.Config(O.DGC, dgc_sample_ppm=10000)
    pay, _ = O.compress(cfg, np.zeros(0, np.float32), np.zeros(0, np.float32))
    assert pay.size == O.HDR and O.header(pay)["k"] == 0
    n = 3000
    cfg = O.Config(O.DGC, ratio_ppm=20000, dgc_momentum=0.9, dgc_sample_ppm=100000, seed=2)
    st = O.new_state(cfg, n)
    g1, g2 = rand_group(n, 1), rand_group(n, 2)
    O.compress(cfg, g1, st, it=0)
    v1, u1 = st[:n].copy(), st[n:].copy()
    pay, _ = O.compress(cfg, g2, st, it=1)
    idx, val = O.sparse_view(pay)
    u = np.float32(0.9) * u1 + g2
    v = v1 + u
    assert np.array_equal(val, v[idx])
    u[idx] = 0
    v[idx] = 0
    assert np.array_equal(st[:n], v) and np.array_equal(st[n:], u)
