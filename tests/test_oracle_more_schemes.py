"""Pins for the oracle's four further schemes of the paper's Table 1: SignSGD, SigNUM, OneBit, Rand-k (CPU only).

The paper only names them (Section 2.1, Table 1).  The oracle's readings are tied down by library routines they
reduce to (numpy packbits, sign of a sum, means, stable argsort), special cases that collapse one scheme into
another, closed forms, the least-squares property of class means, and counting arguments for the random choice.
"""
import numpy as np
import pytest

from oracle import oracle as O


def f32(x):
    return np.asarray(x, dtype=np.float32)


def rand_group(n, seed, scale=1.0):
    return f32(np.random.default_rng(seed).standard_normal(n) * scale)


def bits_of(payload, n):
    return np.unpackbits(payload[O.HDR:O.HDR + 4 * ((n + 31) // 32)], bitorder="little")[:n].astype(bool)


SIZES = [1, 2, 31, 32, 33, 64, 65, 1000, 4097]


# =============================================================== SignSGD ====
@pytest.mark.parametrize("n", SIZES)
def test_signsgd_is_the_packed_sign_and_nothing_else(n):
    cfg = O.Config(O.SIGNSGD, use_ef=0)
    assert O.state_floats(cfg, n) == 0
    g = rand_group(n, n)
    if n > 4:
        g[1] = 0.0
        g[2] = -0.0                      # -0 >= 0: counted as +
    pay, _ = O.compress(cfg, g, None)
    h = O.header(pay)
    assert (h["magic"], h["algo"], h["n"], h["k"], h["scale"]) == (0x3150434D, O.SIGNSGD, n, 0, 1.0)
    assert pay.size == O.HDR + 4 * ((n + 31) // 32)
    want = np.packbits(g >= 0, bitorder="little")
    assert np.array_equal(pay[O.HDR:O.HDR + want.size], want)
    assert not np.unpackbits(pay[O.HDR:], bitorder="little")[n:].any()            # pad bits are 0
    assert np.array_equal(O.decode(pay, n), np.where(g >= 0, np.float32(1), np.float32(-1)))
    # only the signs matter: any positive rescaling gives the same bytes
    pay2, _ = O.compress(cfg, g * np.float32(123.5), None)
    assert np.array_equal(pay, pay2)


def test_signsgd_rejects_error_feedback():
    with pytest.raises(ValueError):
        O.compress(O.Config(O.SIGNSGD, use_ef=1), rand_group(10, 0), None)


@pytest.mark.parametrize("W", [1, 2, 3, 4, 8, 9])
def test_majority_vote_is_the_sign_of_the_sum_of_signs(W):
    n = 777
    cfg = O.Config(O.SIGNSGD, use_ef=0)
    gs = [rand_group(n, 100 + w) for w in range(W)]
    pays = [O.compress(cfg, g, None)[0] for g in gs]
    tally = sum(np.where(g >= 0, 1, -1) for g in gs)                               # integers
    for alpha in (1.0, 0.125, -3.0):
        out = O.decompress_sum(pays, n, alpha)
        assert np.array_equal(out, f32(alpha) * np.sign(tally).astype(np.float32))
    if W % 2 == 0:
        assert (tally == 0).any() and (O.decompress_sum(pays, n)[tally == 0] == 0).all()   # ties vote 0
    else:
        assert (np.abs(O.decompress_sum(pays, n)) == 1).all()


def test_vote_of_identical_workers_is_the_worker():
    g = rand_group(500, 5)
    pay, _ = O.compress(O.Config(O.SIGNSGD, use_ef=0), g, None)
    assert np.array_equal(O.decompress_sum([pay] * 5, 500), O.decode(pay, 500))


# ================================================================ SigNUM ====
def test_signum_with_zero_beta_is_signsgd():
    n = 1500
    for it in range(3):
        g = rand_group(n, 40 + it)
        st = rand_group(n, 50 + it)            # whatever the old momentum was, beta = 0 forgets it
        a, _ = O.compress(O.Config(O.SIGNUM, dgc_momentum=0.0), g, st)
        b, _ = O.compress(O.Config(O.SIGNSGD, use_ef=0), g, None)
        assert np.array_equal(a[O.HDR:], b[O.HDR:])
        assert O.header(a)["algo"] == O.SIGNUM
        assert np.array_equal(st, g)           # m = 0*m + 1*g


def test_signum_momentum_closed_form_for_a_constant_gradient():
    """m_t = (1 - beta^t) g for a constant gradient and m_0 = 0."""
    n, beta = 600, 0.9
    cfg = O.Config(O.SIGNUM, dgc_momentum=beta)
    g = rand_group(n, 8)
    st = O.new_state(cfg, n)
    for t in range(1, 13):
        pay, _ = O.compress(cfg, g, st)
        want = (1.0 - np.float32(beta).astype(np.float64) ** t) * g.astype(np.float64)
        assert np.allclose(st, want, rtol=2e-6, atol=0)
        assert np.array_equal(bits_of(pay, n), g >= 0)


def test_signum_sign_follows_the_momentum_not_the_gradient():
    n, beta = 400, 0.9
    cfg = O.Config(O.SIGNUM, dgc_momentum=beta)
    g = np.abs(rand_group(n, 9)) + np.float32(0.5)
    st = O.new_state(cfg, n)
    for _ in range(10):
        O.compress(cfg, g, st)                         # momentum builds up positive
    pay, _ = O.compress(cfg, -g, st)                   # one opposite gradient does not flip it: 0.9*0.65g - 0.1g > 0
    assert bits_of(pay, n).all()
    m = st.copy()
    for _ in range(40):
        pay, _ = O.compress(cfg, -g, st)
    assert not bits_of(pay, n).any() and (st < 0).all() and (m > 0).all()
    # one step of the recursion against float64 arithmetic
    st2 = m.copy()
    O.compress(cfg, g, st2)
    b = float(np.float32(beta))
    assert np.allclose(st2, b * m.astype(np.float64) + float(np.float32(1) - np.float32(beta)) * g, rtol=3e-7, atol=0)


def test_signum_needs_its_state():
    with pytest.raises(ValueError):
        O.compress(O.Config(O.SIGNUM, use_ef=0), rand_group(10, 0), None)


# ================================================================ OneBit ====
@pytest.mark.parametrize("n", SIZES)
def test_onebit_means_and_reconstruction(n):
    cfg = O.Config(O.ONEBIT)
    g, e0 = rand_group(n, n), rand_group(n, n + 1, 0.3)
    st = e0.copy()
    pay, mu_pos = O.compress(cfg, g, st)
    p = g + e0
    h = O.header(pay)
    pos = p >= 0
    want_pos = np.float32(p[pos].astype(np.float64).mean()) if pos.any() else np.float32(0)
    want_neg = np.float32(p[~pos].astype(np.float64).mean()) if (~pos).any() else np.float32(0)
    assert (h["algo"], h["n"], h["k"]) == (O.ONEBIT, n, 0)
    assert abs(h["scale"] - want_pos) <= 1e-7 * abs(want_pos) and abs(h["scale2"] - want_neg) <= 1e-7 * abs(want_neg)
    assert h["scale"] == mu_pos and h["scale"] >= 0 >= h["scale2"]
    assert np.array_equal(bits_of(pay, n), pos)
    d = O.decode(pay, n)
    assert np.array_equal(d, np.where(pos, np.float32(h["scale"]), np.float32(h["scale2"])))
    assert np.array_equal(st, p - d)                   # residual: one fp32 subtraction
    assert not pay[36:O.HDR].any()                        # rest of the header stays zero


def test_onebit_class_means_preserve_the_sum_and_minimise_the_error():
    n = 20000
    cfg = O.Config(O.ONEBIT)
    p = rand_group(n, 3) + np.float32(0.2)
    st = np.zeros(n, np.float32)
    pay, _ = O.compress(cfg, p, st)
    d = O.decode(pay, n).astype(np.float64)
    pos = p >= 0
    for cls in (pos, ~pos):                            # the residual of each class sums to (almost) zero
        assert abs((p.astype(np.float64)[cls] - d[cls]).sum()) <= 1e-6 * np.abs(p[cls]).sum()
    err = ((p - d) ** 2).sum()
    h = O.header(pay)
    for dp, dn in [(1e-3, 0), (-1e-3, 0), (0, 1e-3), (0, -1e-3)]:      # any other pair of levels does worse
        alt = np.where(pos, h["scale"] + dp, h["scale2"] + dn)
        assert ((p - alt) ** 2).sum() > err


def test_onebit_zeros_belong_to_the_upper_class():
    """The bit of a zero is 1 (p >= 0), so zeros are averaged with the positives."""
    p = f32([0.0, -0.0, 3.0, -1.0, -2.0, 0.0])
    pay, _ = O.compress(O.Config(O.ONEBIT), p, np.zeros(6, np.float32))
    h = O.header(pay)
    assert h["scale"] == np.float32(3.0 / 4.0) and h["scale2"] == np.float32(-1.5)
    assert list(bits_of(pay, 6)) == [True, True, True, False, False, True]


def test_onebit_one_sided_groups_and_scale_override():
    cfg = O.Config(O.ONEBIT)
    p = np.abs(rand_group(100, 4)) + np.float32(1)
    pay, _ = O.compress(cfg, p, np.zeros(100, np.float32))
    assert O.header(pay)["scale2"] == 0.0 and bits_of(pay, 100).all()
    pay, _ = O.compress(cfg, -p, np.zeros(100, np.float32))
    assert O.header(pay)["scale"] == 0.0 and not bits_of(pay, 100).any()
    st = np.zeros(100, np.float32)
    pay, _ = O.compress(cfg, rand_group(100, 6), st, scale_in=(0.5, -0.25))
    assert set(np.unique(O.decode(pay, 100))) == {np.float32(0.5), np.float32(-0.25)}
    assert np.array_equal(st, rand_group(100, 6) - O.decode(pay, 100))


def test_onebit_aggregate_is_the_ordered_sum():
    n, W = 999, 5
    cfg = O.Config(O.ONEBIT)
    pays = [O.compress(cfg, rand_group(n, 60 + w, 1 + w), np.zeros(n, np.float32))[0] for w in range(W)]
    acc = np.zeros(n, np.float32)
    for pay in pays:
        acc = acc + O.decode(pay, n)
    assert np.array_equal(O.decompress_sum(pays, n, 0.2), np.float32(0.2) * acc)


# ================================================================ Rand-k ====
def randk_keys(seed, worker, it, off, n):
    """The selection keys from the Philox block function alone (pinned by its known-answer vectors)."""
    keys = np.empty(n, np.uint32)
    for i in range(n):
        gi = off + i
        J = gi >> 2
        r = O.philox4x32_10([J & 0xFFFFFFFF, J >> 32, worker, it & 0xFFFFFFFF], [seed & 0xFFFFFFFF, seed >> 32])
        keys[i] = r[gi & 3] >> 1
    return keys


@pytest.mark.parametrize("n,ppm,off", [(50, 100000, 0), (1000, 10000, 0), (1000, 250000, 37), (4097, 1000, 2 ** 33 + 1)])
def test_randk_is_the_topk_of_the_philox_keys(n, ppm, off):
    cfg = O.Config(O.RANDK, ratio_ppm=ppm, seed=0x1234567890ABCDEF)
    g, e0 = rand_group(n, 1), rand_group(n, 2, 0.5)
    st = e0.copy()
    pay, _ = O.compress(cfg, g, st, group_off=off, worker=3, it=7)
    k = O.topk_count(n, ppm)
    idx, val = O.sparse_view(pay)
    assert O.header(pay)["k"] == k == idx.size and O.header(pay)["algo"] == O.RANDK
    keys = randk_keys(cfg.seed, 3, 7, off, n)
    assert keys.max() < 2 ** 31
    assert all(O.randk_key(cfg.seed, 3, 7, off + i) == keys[i] for i in range(0, n, 97))
    order = np.argsort(-keys.astype(np.int64), kind="stable")         # key descending, index ascending on ties
    want = np.sort(order[:k])
    assert np.array_equal(idx, want)
    p = g + e0
    assert np.array_equal(val, p[want])
    # conservation: what was sent plus what is remembered is p, exactly
    back = st.copy()
    back[idx] += val
    assert np.array_equal(back, p) and (st[idx] == 0).all()


def test_randk_uses_all_31_key_bits():
    """Two positions whose keys agree in their upper 23 bits: the larger key wins although its index is higher."""
    n, seed = 100000, 0xABCDEF
    keys = np.array([O.randk_key(seed, 0, 0, i) for i in range(n)], dtype=np.uint32)
    order = np.argsort(keys, kind="stable")
    ks = keys[order]
    close = np.nonzero(((ks[1:] >> 8) == (ks[:-1] >> 8)) & (ks[1:] > ks[:-1]) & (order[1:] > order[:-1]))[0]
    assert close.size > 0
    i, j = int(order[close[0]]), int(order[close[0] + 1])          # i < j, key_i < key_j, same upper bits
    k = int((keys >= keys[j]).sum())                               # the threshold falls between the two
    cfg = O.Config(O.RANDK, ratio_ppm=10 * k, seed=seed)
    assert O.topk_count(n, cfg.ratio_ppm) == k
    idx, _ = O.sparse_view(O.compress(cfg, rand_group(n, 1), np.zeros(n, np.float32))[0])
    assert j in idx and i not in idx
    assert np.array_equal(idx, np.sort(np.nonzero(keys >= keys[j])[0]))


def test_randk_choice_ignores_the_values_and_changes_with_worker_and_iteration():
    n = 5000
    cfg = O.Config(O.RANDK, ratio_ppm=20000, seed=11)
    a = O.sparse_view(O.compress(cfg, rand_group(n, 1), np.zeros(n, np.float32), worker=1, it=4)[0])[0]
    b = O.sparse_view(O.compress(cfg, rand_group(n, 2, 100.0), np.zeros(n, np.float32), worker=1, it=4)[0])[0]
    c = O.sparse_view(O.compress(cfg, rand_group(n, 1), np.zeros(n, np.float32), worker=2, it=4)[0])[0]
    d = O.sparse_view(O.compress(cfg, rand_group(n, 1), np.zeros(n, np.float32), worker=1, it=5)[0])[0]
    assert np.array_equal(a, b)
    assert not np.array_equal(a, c) and not np.array_equal(a, d)
    assert (np.diff(a) > 0).all()                       # ascending and distinct


def test_randk_choice_does_not_depend_on_the_partition():
    n = 3000
    cfg = O.Config(O.RANDK, ratio_ppm=1000000, seed=5)    # k = n: everything is kept, keys irrelevant
    g = rand_group(n, 3)
    idx, val = O.sparse_view(O.compress(cfg, g, np.zeros(n, np.float32))[0])
    assert np.array_equal(idx, np.arange(n)) and np.array_equal(val, g)
    # the key of a model element is the same whichever group it falls in
    assert O.randk_key(5, 0, 0, 1234) == randk_keys(5, 0, 0, 1000, 300)[234]


def test_randk_is_uniform_over_positions():
    n, ppm, T = 400, 50000, 600                           # k = 20, each position is hit k/n = 5 % of the time
    cfg = O.Config(O.RANDK, ratio_ppm=ppm, seed=99)
    g = rand_group(n, 1)
    hits = np.zeros(n)
    for it in range(T):
        hits[O.sparse_view(O.compress(cfg, g, np.zeros(n, np.float32), it=it)[0])[0]] += 1
    q = 20 / n
    sigma = np.sqrt(T * q * (1 - q))
    assert np.abs(hits - T * q).max() < 5 * sigma
    assert abs(hits.sum() - 20 * T) == 0


def test_randk_needs_error_feedback_and_sums_like_a_sparsifier():
    with pytest.raises(ValueError):
        O.compress(O.Config(O.RANDK, use_ef=0), rand_group(10, 0), None)
    n, W = 800, 4
    cfg = O.Config(O.RANDK, ratio_ppm=100000, seed=2)
    pays = [O.compress(cfg, rand_group(n, w), np.zeros(n, np.float32), worker=w)[0] for w in range(W)]
    acc = np.zeros(n, np.float32)
    for pay in pays:
        acc = acc + O.decode(pay, n)
    assert np.array_equal(O.decompress_sum(pays, n, 0.25), np.float32(0.25) * acc)


# ============================================================ all four ====
@pytest.mark.parametrize("algo,kw", [(O.SIGNSGD, dict(use_ef=0)), (O.SIGNUM, {}), (O.ONEBIT, {}), (O.RANDK, {})])
def test_empty_and_all_zero_groups(algo, kw):
    cfg = O.Config(algo, **kw)
    pay, _ = O.compress(cfg, np.zeros(0, np.float32), None if algo == O.SIGNSGD else np.zeros(0, np.float32))
    assert pay.size == O.HDR and O.header(pay)["n"] == 0
    n = 300
    st = None if algo == O.SIGNSGD else np.zeros(n, np.float32)
    pay, _ = O.compress(cfg, np.zeros(n, np.float32), st)
    out = O.decompress_sum([pay, pay], n)
    assert np.isfinite(out).all()
    if algo in (O.ONEBIT, O.RANDK):
        assert not out.any()
    else:
        assert (out == 1).all()                          # sign(0) = +, two votes for +
