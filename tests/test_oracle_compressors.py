"""Pins for the oracle's compressors and aggregate (CPU only).

The paper prints no input/output pair for any compressor, so the oracle is tied
down by what the mathematics fixes: library routines it must reduce to (stable
argsort, float16 cast, packbits, norms), brute force on tiny inputs, exact
conservation identities of error feedback, closed forms for the residual
energy, and statistical unbiasedness of the stochastic quantizers.
"""
import math

import numpy as np
import pytest

from oracle import oracle as O


def f32(x):
    return np.asarray(x, dtype=np.float32)


def rand_group(n, seed, scale=1.0):
    rng = np.random.default_rng(seed)
    return f32(rng.standard_normal(n) * scale)


def bits_of(words, n):
    return np.unpackbits(words.view(np.uint8), bitorder="little")[:n].astype(bool)


SIZES = [1, 2, 31, 32, 33, 63, 64, 65, 100, 1000, 4097]


# =============================================================== EF-Sign ====
@pytest.mark.parametrize("n", SIZES)
def test_efsign_decode_is_scale_times_sign(n):
    cfg = O.Config(O.EFSIGN)
    g, e0 = rand_group(n, n), rand_group(n, n + 1, 0.3)
    if n > 4:
        g[3] = 0.0; e0[3] = 0.0          # sign(0) = +1
        g[4] = -0.0; e0[4] = -0.0        # -0 + -0 = -0, still counted as >= 0
    st = e0.copy()
    pay, scale = O.compress(cfg, g, st)
    p = g + e0                           # fp32 add
    h = O.header(pay)
    assert (h["magic"], h["algo"], h["n"], h["k"]) == (0x3150434D, O.EFSIGN, n, 0)
    # scale = mean |p| (library routine, float64), rounded once to fp32
    assert h["scale"] == scale == np.float32(np.abs(p.astype(np.float64)).mean())
    words = pay[O.HDR:].view(np.uint32)
    assert words.size == (n + 31) // 32
    # bit i%32 of word i/32  <->  numpy's little-endian packbits of (p >= 0)
    want = np.packbits(p >= 0, bitorder="little")
    got = words.view(np.uint8)[: want.size]
    assert np.array_equal(got, want)
    assert not np.unpackbits(words.view(np.uint8), bitorder="little")[n:].any()   # pad bits are 0
    d = O.decode(pay, n)
    sgn = np.where(p >= 0, np.float32(1), np.float32(-1))
    assert np.array_equal(d, sgn * np.float32(scale))
    # residual: e = p - d, exactly one fp32 subtraction
    assert np.array_equal(st, p - d)


def test_efsign_residual_energy_closed_form_and_optimal_scale():
    n = 50000
    g = rand_group(n, 11)
    st = np.zeros(n, np.float32)
    pay, scale = O.compress(O.Config(O.EFSIGN), g, st)
    p = g.astype(np.float64)
    l1, l2sq = np.abs(p).sum(), (p * p).sum()
    # ||p - s sign(p)||^2 = ||p||^2 - ||p||_1^2 / n  when s = ||p||_1 / n
    assert np.isclose((st.astype(np.float64) ** 2).sum(), l2sq - l1 * l1 / n, rtol=1e-5)
    # and that s minimises the residual energy: any other scale does worse
    for bad in (0.9, 1.1):
        st2 = np.zeros(n, np.float32)
        O.compress(O.Config(O.EFSIGN), g, st2, scale_in=scale * bad)
        assert (st2.astype(np.float64) ** 2).sum() > (st.astype(np.float64) ** 2).sum()
    # Gaussian input: q = ||Q(x)-x||^2 / ||x||^2 -> 1 - 2/pi  (the paper's q_i, Section 4.2)
    q = (st.astype(np.float64) ** 2).sum() / l2sq
    assert abs(q - (1 - 2 / math.pi)) < 0.01


def test_efsign_error_feedback_telescopes():
    # sum_t decode(payload_t) + e_T == T * g  up to fp32 rounding (constant gradient)
    n, T = 3000, 25
    g = rand_group(n, 5, 0.01)
    st = np.zeros(n, np.float32)
    acc = np.zeros(n, np.float64)
    for t in range(T):
        pay, _ = O.compress(O.Config(O.EFSIGN), g, st, it=t)
        acc += O.decode(pay, n)
    assert np.allclose(acc + st, T * g.astype(np.float64), rtol=0, atol=1e-6)


def test_efsign_scale_override_and_no_ef():
    n = 500
    g = rand_group(n, 2)
    pay, scale = O.compress(O.Config(O.EFSIGN, use_ef=0), g, None, scale_in=0.125)
    assert O.header(pay)["scale"] == 0.125 and scale == np.float32(np.abs(g.astype(np.float64)).mean())
    assert np.array_equal(np.abs(O.decode(pay, n)), np.full(n, 0.125, np.float32))


# ================================================================ Top-k =====
def brute_topk(p, k):
    key = p.view(np.uint32) & np.uint32(0x7FFFFFFF)
    n = p.size
    sel = []
    for i in range(n):
        rank = sum(1 for j in range(n) if key[j] > key[i] or (key[j] == key[i] and j < i))
        if rank < k:
            sel.append(i)
    return np.array(sel, dtype=np.uint32)


def argsort_topk(p, k):
    key = (p.view(np.uint32) & np.uint32(0x7FFFFFFF)).astype(np.int64)
    order = np.argsort(-key, kind="stable")        # library stable sort: ties keep index order
    return np.sort(order[:k]).astype(np.uint32)


TOPK_CASES = [
    ("random", lambda n, r: f32(r.standard_normal(n))),
    ("all_equal", lambda n, r: np.full(n, 0.5, np.float32)),
    ("all_zero", lambda n, r: np.zeros(n, np.float32)),
    ("many_ties", lambda n, r: f32(r.integers(-3, 4, n))),
    ("pm_ties", lambda n, r: f32(r.choice([-1.0, 1.0, 0.25], n))),
    ("single_nonzero", lambda n, r: f32(np.eye(1, n, n // 2)[0] * -7)),
]


@pytest.mark.parametrize("name,gen", TOPK_CASES)
@pytest.mark.parametrize("n", [1, 2, 7, 64, 257])
def test_topk_bruteforce(name, gen, n):
    rng = np.random.default_rng(n)
    p = gen(n, rng)
    for ppm in (1, 10000, 250000, 500000, 10 ** 6):
        cfg = O.Config(O.TOPK, ratio_ppm=ppm)
        k = max(1, n * ppm // 10 ** 6)
        st = np.zeros(n, np.float32)
        pay, _ = O.compress(cfg, p, st)
        p = p + st * 0                                                  # what is compressed is g + e (e = +0)
        idx, val = O.sparse_view(pay)
        h = O.header(pay)
        assert h["k"] == k == idx.size == O.topk_count(n, ppm)          # exact-k
        assert np.array_equal(idx, brute_topk(p, k))
        assert np.array_equal(idx, argsort_topk(p, k))
        assert np.all(np.diff(idx.astype(np.int64)) > 0)                # ascending, unique
        assert np.array_equal(val.view(np.uint32), p[idx].view(np.uint32))  # values are bit copies


@pytest.mark.parametrize("n,ppm", [(5000, 10000), (100000, 1000), (40000, 10000), (4097, 500000)])
def test_topk_argsort_and_conservation(n, ppm):
    rng = np.random.default_rng(n + ppm)
    g = f32(rng.standard_normal(n) * 10.0 ** rng.uniform(-4, -1, n))
    g[::7] = np.float32(0.03125)          # plant many exact ties around the threshold region
    e0 = rand_group(n, 99, 0.01)
    st = e0.copy()
    pay, _ = O.compress(O.Config(O.TOPK, ratio_ppm=ppm), g, st)
    p = g + e0
    idx, val = O.sparse_view(pay)
    k = O.topk_count(n, ppm)
    assert idx.size == k
    assert np.array_equal(idx, argsort_topk(p, k))
    # conservation: scatter(payload) + e_new == g + e_old, element-wise and exactly
    dense = O.decode(pay, n)
    assert np.array_equal((dense + st).view(np.uint32), (p + np.float32(0)).view(np.uint32))
    assert np.all(st[idx] == 0) and np.array_equal(dense[idx], p[idx])
    # energy identity
    assert np.isclose((st.astype(np.float64) ** 2).sum(),
                      (p.astype(np.float64) ** 2).sum() - (val.astype(np.float64) ** 2).sum(), rtol=1e-9)
    # every kept magnitude >= every dropped magnitude
    mask = np.ones(n, bool); mask[idx] = False
    if mask.any():
        assert np.abs(p[idx]).min() >= np.abs(p[mask]).max()


def test_topk_without_error_feedback_and_empty_group():
    g = rand_group(1000, 4)
    pay, _ = O.compress(O.Config(O.TOPK, use_ef=0, ratio_ppm=50000), g, None)
    idx, val = O.sparse_view(pay)
    assert np.array_equal(idx, argsort_topk(g, 50)) and np.array_equal(val, g[idx])
    pay, _ = O.compress(O.Config(O.TOPK), np.zeros(0, np.float32), np.zeros(0, np.float32))
    assert pay.size == O.HDR and O.header(pay)["k"] == 0 and O.header(pay)["n"] == 0


# ================================================================== DGC =====
def test_dgc_zero_momentum_is_topk():
    n = 20000
    st_t = np.zeros(n, np.float32)
    st_d = np.zeros(2 * n, np.float32)
    for t in range(4):
        g = rand_group(n, 100 + t, 0.02)
        pt, _ = O.compress(O.Config(O.TOPK, ratio_ppm=5000), g, st_t, it=t)
        pd, _ = O.compress(O.Config(O.DGC, ratio_ppm=5000, dgc_momentum=0.0), g, st_d, it=t)
        assert O.header(pd)["algo"] == O.DGC
        assert np.array_equal(pt[8:], pd[8:])                  # all but magic/algo
        assert np.array_equal(st_t.view(np.uint32), st_d[:n].view(np.uint32))


def test_dgc_conservation_and_masking():
    n, m = 30000, np.float32(0.9)
    st = np.zeros(2 * n, np.float32)
    for t in range(3):
        g = rand_group(n, 200 + t, 0.02)
        v_old, u_old = st[:n].copy(), st[n:].copy()
        pay, _ = O.compress(O.Config(O.DGC, ratio_ppm=1000), g, st, it=t)
        u_new = m * u_old + g                                   # two fp32 roundings: mul then add
        v_acc = v_old + u_new
        idx, val = O.sparse_view(pay)
        assert idx.size == 30
        assert np.array_equal(idx, argsort_topk(v_acc, 30))
        assert np.array_equal(val.view(np.uint32), v_acc[idx].view(np.uint32))
        dense = O.decode(pay, n)
        assert np.array_equal(dense + st[:n], v_acc + np.float32(0))
        keep = np.ones(n, bool); keep[idx] = False
        assert np.array_equal(st[n:][keep], u_new[keep]) and np.all(st[n:][idx] == 0) and np.all(st[:n][idx] == 0)


def test_dgc_momentum_closed_form():
    # an entry that is never selected accumulates u_T = g (1 - m^T)/(1 - m), v_T = sum_t u_t
    n, T, m = 2000, 6, 0.9
    g = np.full(n, 0.001, np.float32)
    g[0] = 1.0                                  # index 0 is taken every time (k = 1)
    st = np.zeros(2 * n, np.float32)
    for t in range(T):
        pay, _ = O.compress(O.Config(O.DGC, ratio_ppm=1, dgc_momentum=m), g, st, it=t)
        assert list(O.sparse_view(pay)[0]) == [0]
    u = [0.001 * (1 - m ** (t + 1)) / (1 - m) for t in range(T)]
    assert np.allclose(st[n + 1:], u[-1], rtol=1e-5)
    assert np.allclose(st[1:n], sum(u), rtol=1e-5)
    with pytest.raises(ValueError):
        O.compress(O.Config(O.DGC, use_ef=0), g, None)


def test_sparse_payload_ends_with_a_directory_of_its_index_list():
    """Entry t of the directory counts the kept entries with index below 4096 t (a library search over the index list is
    the reference); payload size = header + 8 k + 4 (spans + 1).  Exact top-k, DGC, Rand-k and DGC with a capacity."""
    n = 3 * 4096 + 77
    g = rand_group(n, 71, 0.1)
    g[4096:2 * 4096] *= 1e-4                      # a span with no kept entry
    for cfg in (O.Config(O.TOPK, ratio_ppm=20000), O.Config(O.DGC, ratio_ppm=20000), O.Config(O.RANDK, ratio_ppm=20000, seed=3),
                O.Config(O.DGC, ratio_ppm=20000, dgc_sample_ppm=100000, seed=5)):
        pay, _ = O.compress(cfg, g, O.new_state(cfg, n), worker=1, it=2)
        idx, _ = O.sparse_view(pay)
        h = O.header(pay)
        cap = h["levels"] or h["k"]
        spans = (n + 4095) // 4096
        assert pay.size == O.HDR + 8 * cap + 4 * (spans + 1) == O.payload_bytes(cfg, n)
        d = O.sparse_directory(pay)
        assert d.size == spans + 1 and d[0] == 0 and d[-1] == h["k"] == idx.size
        assert np.array_equal(d, np.searchsorted(idx, np.arange(spans + 1) * 4096, side="left"))
        if cfg.algo != O.RANDK and not cfg.dgc_sample_ppm:
            assert d[2] == d[1]                       # nothing kept in the quiet span
        # what a payload built from the lists alone looks like (the helper the GPU tests use)
        if not cfg.dgc_sample_ppm:
            assert np.array_equal(O.with_directory(cfg.algo, n, idx, O.sparse_view(pay)[1]), pay)


# ================================================================= QSGD =====
def test_qsgd_structure():
    n = 5000
    g, e0 = rand_group(n, 21, 0.05), rand_group(n, 22, 0.01)
    g[:3] = 0; e0[:3] = 0
    for bits in (8, 4, 2):
        s = 2 ** (bits - 1) - 1
        st = e0.copy()
        pay, norm = O.compress(O.Config(O.QSGD, qsgd_bits=bits, seed=3), g, st, worker=1, it=2)
        p = g + e0
        h = O.header(pay)
        assert h["levels"] == s and h["scale"] == norm == np.float32(np.linalg.norm(p.astype(np.float64)))
        code = pay[O.HDR:O.HDR + n].view(np.int8).astype(np.int64)
        assert np.abs(code).max() <= s and np.all(code[:3] == 0)            # range; 0 -> code 0
        assert np.all((code < 0) <= (p < 0)) and np.all((code > 0) <= (p > 0))   # sign follows p
        # the level is one of the two integers bracketing |p| s / norm
        a = np.abs(p.astype(np.float64)) * s / float(norm)
        assert np.all(np.abs(code) >= np.floor(a - 1e-4)) and np.all(np.abs(code) <= np.floor(a + 1e-4) + 1)
        d = O.decode(pay, n)
        assert np.array_equal(d, code.astype(np.float32) * (np.float32(norm) / np.float32(s)))
        assert np.array_equal(st, p - d)
        assert np.all(np.abs(st.astype(np.float64)) <= float(norm) / s * (1 + 1e-5))


def _average_decode(cfg_of_seed, g, T):
    acc = np.zeros(g.size, np.float64)
    sq = 0.0
    for t in range(T):
        pay, _ = O.compress(cfg_of_seed(t), g, None)
        d = O.decode(pay, g.size).astype(np.float64)
        acc += d
        sq += (d * d).sum()
    return acc / T, sq / T


def test_qsgd_unbiased_by_averaging():
    n, T, s = 48, 3000, 127
    g = rand_group(n, 31, 0.1)
    mean, _ = _average_decode(lambda t: O.Config(O.QSGD, use_ef=0, seed=1000 + t), g, T)
    p = g.astype(np.float64)
    norm = np.linalg.norm(p)
    a = np.abs(p) * s / norm
    f = a - np.floor(a)
    sigma = norm / s * np.sqrt(f * (1 - f))                 # Bernoulli between adjacent levels
    assert np.all(np.abs(mean - p) <= 5 * sigma / math.sqrt(T) + 1e-7)
    # a biased rounding rule (always down / nearest) would be off by O(norm/s): make sure we could see it
    assert (5 * sigma / math.sqrt(T)).max() < 0.2 * norm / s


def test_qsgd_low_bit_unbiased():
    n, T, s = 16, 4000, 1
    g = rand_group(n, 33, 1.0)
    mean, _ = _average_decode(lambda t: O.Config(O.QSGD, use_ef=0, qsgd_bits=2, seed=t), g, T)
    p = g.astype(np.float64); norm = np.linalg.norm(p)
    a = np.abs(p) / norm
    assert np.all(np.abs(mean - p) <= 5 * norm * np.sqrt(a * (1 - a) / T) + 1e-7)


# ============================================================= TernGrad =====
def test_terngrad_structure():
    n = 3000
    g = rand_group(n, 41, 0.05)
    g[5] = 0.0
    st = np.zeros(n, np.float32)
    pay, smax = O.compress(O.Config(O.TERNGRAD, seed=9), g, st)
    assert smax == np.abs(g).max() == O.header(pay)["scale"]
    W = (n + 31) // 32
    body = pay[O.HDR:].view(np.uint32)
    assert body.size == 2 * W
    nz, neg = bits_of(body[:W].copy(), n), bits_of(body[W:].copy(), n)
    assert np.all(neg <= nz) and np.array_equal(neg, nz & (g < 0))
    assert nz[int(np.argmax(np.abs(g)))] and not nz[5]       # |p| = smax always kept, 0 never
    d = O.decode(pay, n)
    assert np.array_equal(d, np.where(nz, np.where(neg, -smax, smax), 0).astype(np.float32))
    assert np.array_equal(st, g - d)
    # the Bernoulli draw is [u * smax < |p|] with u the element's Philox uniform
    u = f32([O.uniform(9, 0, 0, i) for i in range(n)])
    assert np.array_equal(nz, (u * np.float32(smax)) < np.abs(g))


def test_terngrad_unbiased_and_second_moment():
    n, T = 40, 4000
    g = rand_group(n, 43, 0.2)
    mean, sq = _average_decode(lambda t: O.Config(O.TERNGRAD, use_ef=0, seed=500 + t), g, T)
    p = g.astype(np.float64); smax = np.abs(p).max()
    sigma = np.sqrt(np.abs(p) * (smax - np.abs(p)))
    assert np.all(np.abs(mean - p) <= 5 * sigma / math.sqrt(T) + 1e-7)
    # E||d||^2 = smax * ||p||_1
    assert abs(sq / (smax * np.abs(p).sum()) - 1) < 0.02


def test_stochastic_draws_do_not_depend_on_partition():
    n, cut = 1000, 372          # cut not a multiple of 4: Philox blocks straddle the boundary
    g = rand_group(n, 51, 0.1)
    cfg = O.Config(O.TERNGRAD, use_ef=0, seed=77)
    smax = float(np.abs(g).max())
    whole, _ = O.compress(cfg, g, None, worker=3, it=5, scale_in=smax)
    a, _ = O.compress(cfg, g[:cut], None, group_off=0, worker=3, it=5, scale_in=smax)
    b, _ = O.compress(cfg, g[cut:], None, group_off=cut, worker=3, it=5, scale_in=smax)
    assert np.array_equal(O.decode(whole, n), np.concatenate([O.decode(a, cut), O.decode(b, n - cut)]))
    other, _ = O.compress(cfg, g, None, worker=4, it=5, scale_in=smax)
    assert not np.array_equal(O.decode(whole, n), O.decode(other, n))


def test_qsgd_draw_is_the_elements_own_philox_uniform():
    """Which draw an element rounds with: the Philox uniform of (seed, worker, iteration, model-global index), the keying
    of the random streams that the benchmark fixes ("keyed on (seed, worker, element)").  The level rule is retyped here
    on top of O.uniform, whose counter / key layout the published Philox vectors and test_uniform_range_mean_and_keying
    pin; group_off is no multiple of 4, worker and iteration are not 0, so a draw that drops any of them differs."""
    n, goff, worker, it, seed, s = 3001, 1234567 * 4 + 3, 5, 9, 0x1234567890ABCDEF, 127
    g = rand_group(n, 61, 0.05)
    pay, norm = O.compress(O.Config(O.QSGD, use_ef=0, seed=seed), g, None, group_off=goff, worker=worker, it=it)
    code = pay[O.HDR:O.HDR + n].view(np.int8).astype(np.int64)
    r = np.float32(s) / np.float32(norm)
    a = np.abs(g) * r                                  # fp32 product, as the rule states it
    lo = np.floor(a)
    frac = (a - lo).astype(np.float32)

    def levels(w, i, off):
        u = f32([O.uniform(seed, w, i, off + j) for j in range(n)])
        return np.minimum(lo.astype(np.int64) + (u < frac), s)

    want = levels(worker, it, goff)
    assert np.array_equal(np.abs(code), want)
    # the check can tell the streams apart: dropping the worker, the iteration or the group's offset changes levels
    for w, i, off in ((0, it, goff), (worker, 0, goff), (worker, it, 0), (worker, it, goff - 3), (0, 0, 0)):
        assert not np.array_equal(levels(w, i, off), want), (w, i, off)


def test_qsgd_draws_do_not_depend_on_partition():
    n, cut = 1000, 373          # cut not a multiple of 4: Philox blocks straddle the boundary
    g = rand_group(n, 53, 0.1)
    cfg = O.Config(O.QSGD, use_ef=0, seed=78)
    norm = float(np.float32(np.linalg.norm(g.astype(np.float64))))
    whole, _ = O.compress(cfg, g, None, group_off=8, worker=3, it=5, scale_in=norm)
    a, _ = O.compress(cfg, g[:cut], None, group_off=8, worker=3, it=5, scale_in=norm)
    b, _ = O.compress(cfg, g[cut:], None, group_off=8 + cut, worker=3, it=5, scale_in=norm)
    assert np.array_equal(whole[O.HDR:O.HDR + n], np.concatenate([a[O.HDR:O.HDR + cut], b[O.HDR:O.HDR + n - cut]]))
    for kw in (dict(worker=4, it=5), dict(worker=3, it=6)):
        other, _ = O.compress(cfg, g, None, group_off=8, scale_in=norm, **kw)
        assert not np.array_equal(whole[O.HDR:O.HDR + n], other[O.HDR:O.HDR + n])


@pytest.mark.parametrize("algo", [O.EFSIGN, O.TOPK, O.DGC, O.QSGD, O.TERNGRAD, O.FP16])
def test_all_zero_group_gives_zero_output(algo):
    n = 100
    cfg = O.Config(algo)
    st = O.new_state(cfg, n)
    pay, scale = O.compress(cfg, np.zeros(n, np.float32), st)
    d = O.decode(pay, n)
    assert scale == 0 and np.all(d == 0) and np.all(np.isfinite(d)) and np.all(st == 0)
    if algo not in (O.EFSIGN, O.TOPK, O.DGC):       # (sign bits of +0 are 1; sparsifiers list k indices)
        assert not pay[O.HDR:].any()                # all-zero group -> all-zero payload body


# ================================================================= FP16 =====
def test_fp16_matches_library_cast():
    specials = f32([0.0, -0.0, 65504.0, 65519.9, 65520.0, -65520.0, 1e9, 2.0 ** -14, 2.0 ** -24, 2.0 ** -25,
                    np.nextafter(np.float32(2.0 ** -25), np.float32(1)), 3 * 2.0 ** -25, 2.0 ** -26, 1.0009765625,
                    1.00048828125, 1.00146484375, 6.1e-5, -5.97e-8, 1e-40])
    rng = np.random.default_rng(0)
    x = np.concatenate([specials, f32(rng.standard_normal(200000) * 10.0 ** rng.integers(-9, 6, 200000))])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16)
    assert np.array_equal(O.f32_to_f16_bits(x), want.view(np.uint16))
    # all 65536 half patterns decode like the library (NaNs compared as NaN)
    allh = np.arange(65536, dtype=np.uint16)
    got, ref = O.f16_bits_to_f32(allh), allh.view(np.float16).astype(np.float32)
    assert np.array_equal(got[~np.isnan(ref)], ref[~np.isnan(ref)]) and np.all(np.isnan(got[np.isnan(ref)]))


def test_fp16_compress_residual_exact():
    n = 10001
    g, e0 = rand_group(n, 61, 0.01), rand_group(n, 62, 1e-5)
    st = e0.copy()
    pay, _ = O.compress(O.Config(O.FP16), g, st)
    p = g + e0
    assert pay.size == O.HDR + (2 * n + 3) // 4 * 4
    h = pay[O.HDR:O.HDR + 2 * n].view(np.float16)
    assert np.array_equal(h.view(np.uint16), p.astype(np.float16).view(np.uint16))
    d = O.decode(pay, n)
    assert np.array_equal(d, h.astype(np.float32))
    # the rounding error of the cast is itself an fp32 number: e + d == p exactly, in any precision
    assert np.array_equal(st.astype(np.float64) + d.astype(np.float64), p.astype(np.float64))


# ============================================================ aggregate =====
def _payloads(cfg, n, W, seed):
    out = []
    for w in range(W):
        st = O.new_state(cfg, n)
        pay, _ = O.compress(cfg, rand_group(n, seed + w, 0.05), st, worker=w)
        out.append(pay)
    return out


@pytest.mark.parametrize("algo", [O.EFSIGN, O.TOPK, O.DGC, O.QSGD, O.TERNGRAD, O.FP16])
def test_aggregate_against_python_loop(algo):
    n, W = 333, 5
    cfg = O.Config(algo, ratio_ppm=100000)
    pays = _payloads(cfg, n, W, 700)
    one = O.decompress_sum(pays[:1], n)
    assert np.array_equal(one, O.decode(pays[0], n) + np.float32(0))        # W = 1, alpha = 1
    out = O.decompress_sum(pays, n, alpha=0.25)
    dec = [O.decode(p, n) for p in pays]
    for i in range(n):                                                     # sequential fp32, ascending worker
        acc = np.float32(0)
        for w in range(W):
            acc = np.float32(acc + dec[w][i])
        assert out[i] == np.float32(np.float32(0.25) * acc)
    # worker order only matters within rounding
    perm = O.decompress_sum(pays[::-1], n, alpha=0.25)
    mag = 0.25 * np.sum([np.abs(d) for d in dec], axis=0)
    assert np.all(np.abs(perm - out) <= 1e-6 * mag + 1e-30)


def test_sparse_aggregate_overlapping_indices():
    n = 64
    cfg = O.Config(O.TOPK, use_ef=0, ratio_ppm=250000)
    base = np.zeros(n, np.float32); base[:16] = np.arange(16, 0, -1)
    pays = [O.compress(cfg, base * np.float32(w + 1), None)[0] for w in range(3)]
    out = O.decompress_sum(pays, n)
    assert np.array_equal(out[:16], base[:16] * 6) and np.all(out[16:] == 0)


def test_decode_rejects_mismatched_payload():
    pay, _ = O.compress(O.Config(O.EFSIGN, use_ef=0), rand_group(64, 1), None)
    with pytest.raises(ValueError):
        O.decode(pay, 65)
    bad = pay.copy(); bad[0] ^= 0xFF
    with pytest.raises(ValueError):
        O.decompress_sum([bad], 64)
