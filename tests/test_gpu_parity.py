"""GPU-vs-oracle parity through the C ABI (run with -m gpu on an MI355X).

Small configurations (the MLP and ResNet-20-shaped sets, and hand-made edge
cases) are compared element by element for every (iteration, group, worker).
The full-size configurations live in test_gpu_fullsize.py.
"""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2103_15195_amd import binding as B
from paper_2103_15195_amd import workloads as WL

import harness as H

pytestmark = pytest.mark.gpu

ALL = ["efsign", "topk", "dgc", "qsgd", "terngrad", "fp16", "signsgd", "signum", "onebit", "randk"]
_cache = {}


def normal_grads(total, seed, scale=0.01):
    def fn(w, it):
        rng = np.random.default_rng([seed, w, it])
        return (rng.standard_normal(total, dtype=np.float32) * np.float32(scale))
    return fn


# ---- first benchmark configuration: MLP, y=2, W=4, EF-Sign and Top-k 1 %, 3 iterations ----------
@pytest.mark.parametrize("algo", ["efsign", "topk"])
def test_config0_mlp(algo):
    wl = WL.workload(0)
    st = H.run_parity(wl.numel, algo, 2, 4, 3, H.workload_grads(wl, cache=_cache), ratio_ppm=10000)
    assert st.compress_checks == 3 * 2 * 4 and st.decompress_checks == 2
    print(f"[config0 {algo}] conditional re-encodes: {st.conditional}")


# ---- second benchmark configuration: ResNet-20 shapes, y in {1,2,4,8,16}, W=8, all algorithms
# (the six of the benchmark and the four further schemes of the paper's Table 1) ------
@pytest.mark.parametrize("y", [1, 2, 4, 8, 16])
@pytest.mark.parametrize("algo", ALL)
def test_config1_resnet20(algo, y):
    wl = WL.workload(1)
    st = H.run_parity(wl.numel, algo, y, 8, 2, H.workload_grads(wl, cache=_cache), ratio_ppm=10000, seed=1234)
    assert st.compress_checks == 2 * y * 8 and st.decompress_checks == y
    print(f"[config1 {algo} y={y}] conditional re-encodes: {st.conditional}")


def test_config1_even_count_partition_and_shared_entries():
    wl = WL.workload(1)
    for algo in ("topk", "dgc", "efsign"):
        H.run_parity(wl.numel, algo, 4, 8, 2, H.workload_grads(wl, shared_fraction=0.8), policy=B.MC_PART_EVEN_COUNT,
                     ratio_ppm=1000 if algo == "dgc" else 10000)


# ---- ragged sizes, tile boundaries, tiny tensors, unaligned tensors -------------------------
RAGGED = [
    [1], [63], [64], [65], [1023], [1024], [1025], [4095], [4096], [4097], [12289],
    [3, 1, 1, 2], [10, 2560, 256, 65536, 7, 1000, 91], [5, 0, 0, 1031, 0, 2],
    [33] * 130,                    # many small tensors inside one chunk
    [7] * 300 + [0, 3, 0] * 20 + [2000],     # more than 64 tensors inside one chunk (the tensor loop takes them 64 at a time)
    [4096, 1, 4095, 8191],
]


@pytest.mark.parametrize("algo", ALL)
@pytest.mark.parametrize("layout", ["separate", "misaligned"])
def test_ragged_and_unaligned(algo, layout):
    for numel in RAGGED:
        total = sum(numel)
        for y in sorted({1, min(2, len(numel)), len(numel) if len(numel) <= 6 else 3}):
            H.run_parity(numel, algo, y, 3, 2, normal_grads(total, seed=total + y), layout=layout,
                         ratio_ppm=100000, seed=99, alpha=0.5)


@pytest.mark.parametrize("algo", ["efsign", "topk", "qsgd", "fp16"])
def test_thousands_of_tensors(algo):
    """6000 tensors of 0..2000 elements, each its own allocation: the address list of a group is uploaded in many
    pieces, most chunks straddle tensors, and a chunk can hold more tensors than a wavefront has lanes."""
    rng = np.random.default_rng(6000)
    numel = rng.integers(0, 2001, 6000)
    numel[rng.integers(0, 6000, 600)] = rng.integers(0, 8, 600)       # runs of tiny and empty tensors
    numel[1000:1200] = rng.integers(0, 4, 200)
    numel = numel.tolist()
    st = H.run_parity(numel, algo, 3, 2, 2, normal_grads(sum(numel), seed=60), ratio_ppm=10000, seed=6, alpha=0.5)
    assert st.compress_checks == 2 * 3 * 2


@pytest.mark.parametrize("algo", ALL)
def test_groups_made_of_empty_tensors(algo):
    numel = [0, 0, 100, 0, 5000, 0]
    H.run_parity(numel, algo, 3, 2, 2, normal_grads(5100, seed=3), user_bounds=[0, 2, 4, 6], policy=B.MC_PART_USER,
                 ratio_ppm=20000)


# ---- degenerate values ------------------------------------------------------------------------
def special_grads(total, kind):
    def fn(w, it):
        rng = np.random.default_rng([17, w, it])
        if kind == "zeros":
            return np.zeros(total, np.float32)
        if kind == "all_equal":
            return np.full(total, 0.25 * (1 if (w + it) % 2 else -1), np.float32)
        if kind == "ties":
            return rng.integers(-3, 4, total).astype(np.float32) * np.float32(0.125)
        if kind == "tiny":        # fp32 subnormals and values below the smallest fp16 subnormal
            return (rng.standard_normal(total, dtype=np.float32) * np.float32(1e-41)).astype(np.float32)
        if kind == "fp16_edges":
            base = np.array([65504.0, 65519.9, 65520.0, -65520.0, 1e9, 2.0 ** -14, 2.0 ** -24, 2.0 ** -25, 3 * 2.0 ** -25,
                             2.0 ** -26, 1.0009765625, 1.00048828125, 1.00146484375, 6.1e-5, -5.97e-8, 0.0, -0.0], np.float32)
            return np.resize(base, total) * np.float32(1 if it == 0 else 0.5)
        if kind == "wide":        # magnitudes over 30 decades
            return (rng.standard_normal(total, dtype=np.float32) * (10.0 ** rng.uniform(-25, 5, total)).astype(np.float32))
        raise ValueError(kind)
    return fn


@pytest.mark.parametrize("kind", ["zeros", "all_equal", "ties", "tiny", "wide"])
@pytest.mark.parametrize("algo", ALL)
def test_degenerate_values(algo, kind):
    numel = [3000, 17, 5000, 1200]
    H.run_parity(numel, algo, 2, 3, 3, special_grads(sum(numel), kind), ratio_ppm=30000, seed=5)


def test_fp16_edge_values():
    H.run_parity([4099], "fp16", 1, 2, 2, special_grads(4099, "fp16_edges"))


@pytest.mark.parametrize("ppm", [1, 500, 500000, 1000000])
@pytest.mark.parametrize("algo", ["topk", "dgc"])
def test_sparsifier_ratios(algo, ppm):
    numel = [20000, 333, 4096]
    H.run_parity(numel, algo, 1, 3, 2, special_grads(sum(numel), "ties" if ppm >= 500000 else "wide"), ratio_ppm=ppm)
    H.run_parity(numel, algo, 2, 2, 2, normal_grads(sum(numel), seed=ppm), ratio_ppm=ppm)


@pytest.mark.parametrize("algo", ["topk", "qsgd", "terngrad", "efsign", "fp16", "onebit"])
def test_without_error_feedback(algo):
    numel = [7000, 129, 4096]
    H.run_parity(numel, algo, 2, 3, 2, normal_grads(sum(numel), seed=8), use_ef=0, ratio_ppm=20000, seed=11)


@pytest.mark.parametrize("algo", ["topk", "dgc"])
@pytest.mark.parametrize("use_ef", [1, 0])
def test_sparsifier_when_the_candidate_filter_misses(algo, use_ef):
    """The candidate filter is seeded by the previous call's threshold.  Gradients that shrink by orders of
    magnitude between calls (over iterations, and between the workers that share a context) leave fewer than k
    candidates and force the refill path; growing ones make nearly everything a candidate.  Results stay exact."""
    if algo == "dgc" and not use_ef:
        pytest.skip("DGC always carries state")
    numel = [30000, 17, 5000, 12000]
    total = sum(numel)

    def grads(w, it):
        rng = np.random.default_rng([23, w, it])
        scale = [1.0, 1e-3, 10.0, 1e-6, 1e-6, 1.0][it] * (1.0 if w % 2 == 0 else 1e-2)
        return rng.standard_normal(total, dtype=np.float32) * np.float32(scale)
    H.run_parity(numel, algo, 2, 3, 6, grads, ratio_ppm=10000, use_ef=use_ef, dgc_momentum=0.5)
    H.run_parity(numel, algo, 1, 2, 6, grads, ratio_ppm=300000, use_ef=use_ef, dgc_momentum=0.5)


# ---- DGC with a threshold taken from a sample: variable number of kept entries, capacity 2k ---------------
@pytest.mark.parametrize("sample_ppm", [1000000, 200000, 10000, 1000])
def test_dgc_sampled_threshold(sample_ppm):
    numel = [30000, 17, 5000, 12000, 1]
    total = sum(numel)
    for y, W in ((1, 3), (2, 2), (5, 2)):
        st = H.run_parity(numel, "dgc", y, W, 3, normal_grads(total, seed=sample_ppm + y), ratio_ppm=20000, dgc_momentum=0.7,
                          dgc_sample_ppm=sample_ppm, seed=31)
        assert st.decompress_checks == y


@pytest.mark.parametrize("kind", ["zeros", "all_equal", "ties", "wide"])
def test_dgc_sampled_threshold_on_degenerate_values(kind):
    """Tied values make far more than k elements reach the sampled threshold: the capacity rule decides."""
    numel = [3000, 17, 5000, 1200]
    H.run_parity(numel, "dgc", 2, 3, 3, special_grads(sum(numel), kind), ratio_ppm=30000, dgc_sample_ppm=50000, seed=5)
    H.run_parity([4097], "dgc", 1, 2, 2, special_grads(4097, kind), ratio_ppm=500000, dgc_sample_ppm=100000, seed=6)


def test_dgc_sampled_threshold_when_the_hint_misses():
    numel = [30000, 17, 5000, 12000]
    total = sum(numel)

    def grads(w, it):
        rng = np.random.default_rng([29, w, it])
        scale = [1.0, 1e-3, 10.0, 1e-6, 1e-6, 1.0][it]
        return rng.standard_normal(total, dtype=np.float32) * np.float32(scale)
    H.run_parity(numel, "dgc", 2, 2, 6, grads, ratio_ppm=10000, dgc_momentum=0.3, dgc_sample_ppm=100000, seed=8)


@pytest.mark.parametrize("algo", ALL)
def test_non_finite_gradients_leave_the_context_usable(algo):
    """Codes of non-finite values are unspecified, but such a call must end normally and what it leaves in the
    context (candidate-filter hints, histograms, tables) must not change later results."""
    numel = [5000, 77, 3000]

    def poisoned(w):
        g = normal_grads(8077, seed=70 + w)(w, 0)
        g[w::97] = np.float32("nan")
        g[5::131] = np.float32("inf")
        g[9::89] = np.float32("-inf")
        return g
    H.run_parity(numel, algo, 1, 2, 2, normal_grads(8077, seed=71), ratio_ppm=20000, prelude_fn=poisoned)


@pytest.mark.parametrize("algo", ["efsign", "topk", "qsgd"])
def test_on_a_stream_of_the_caller(algo):
    """All work is enqueued on the stream that the caller names (here: not the default one)."""
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        st = H.run_parity([5000, 77, 3000], algo, 2, 3, 2, normal_grads(8077, seed=72), ratio_ppm=20000)
    side.synchronize()
    assert st.compress_checks == 2 * 2 * 3


@pytest.mark.parametrize("bits", [2, 4, 7])
def test_qsgd_code_widths(bits):
    H.run_parity([9000, 100], "qsgd", 1, 2, 2, normal_grads(9100, seed=bits), qsgd_bits=bits, seed=21)


def test_dgc_momentum_values():
    for m in (0.0, 0.5, 0.99):
        H.run_parity([9000, 100, 3000], "dgc", 2, 2, 4, normal_grads(12100, seed=4), dgc_momentum=m, ratio_ppm=5000)


@pytest.mark.parametrize("W", [1, 2, 17, 64])
@pytest.mark.parametrize("algo", ALL)
def test_worker_counts(algo, W):
    H.run_parity([5000, 77], algo, 1, W, 1, normal_grads(5077, seed=W), ratio_ppm=50000, alpha=1.0 / W)


@pytest.mark.parametrize("algo", ["qsgd", "terngrad", "randk", "topk", "dgc"])
def test_worker_and_iteration_numbers_beyond_the_usual(algo):
    """Worker numbers that share a hint record (equal modulo 64) or do not fit 31 bits, iteration numbers around
    2^32 (the random stream takes their low word): the random draws follow the oracle's, and a shared hint never
    changes a result."""
    ids = [0, 64, 128, (1 << 31) + 5, (1 << 32) - 1]
    H.run_parity([5000, 77, 4096], algo, 2, len(ids), 3, normal_grads(9173, seed=31), ratio_ppm=20000, seed=(1 << 63) + 12345,
                 worker_id=lambda w: ids[w], iter0=(1 << 32) - 2)


# ---- determinism, state conversion, error reporting ------------------------------------------
@pytest.mark.parametrize("algo", ALL)
def test_bit_reproducible_runs(algo):
    wl = WL.workload(1)
    numel = wl.numel.tolist()
    flat = WL.gradients_flat(wl, 0, 0)
    results = []
    for rep in range(2):
        ctx = B.Context(algo, numel, B.mc_partition(numel, 2), ratio_ppm=10000, seed=3)
        dev = H.device_tensors(flat, numel)
        out = []
        states = [torch.zeros(ctx.state_bytes(g), dtype=torch.uint8, device=H.DEV) for g in range(2)]
        for it in range(2):
            for j in range(2):
                pay = torch.zeros(ctx.payload_bytes(j), dtype=torch.uint8, device=H.DEV)
                ctx.mc_compress(j, 0, it, dev[ctx.bounds[j]:ctx.bounds[j + 1]], states[j], pay)
                out.append(pay.cpu().numpy())
        out += [s.cpu().numpy() for s in states]
        results.append(out)
        ctx.close()
    for a, b in zip(*results):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("algo", ALL)
def test_state_import_export_roundtrip(algo):
    if algo == "signsgd":
        pytest.skip("SignSGD keeps no state")
    n = 10007
    ctx = B.Context(algo, [n], [0, 1], ratio_ppm=10000)
    nf = n * (2 if algo == "dgc" else 1)
    rng = np.random.default_rng(1)
    e = rng.standard_normal(nf, dtype=np.float32)
    e[:4] = [0.0, -0.0, 1e-42, -1e-42]
    state = torch.full((ctx.state_bytes(0),), 0x55, dtype=torch.uint8, device=H.DEV)
    back = torch.zeros(nf, dtype=torch.float32, device=H.DEV)
    ctx.mc_state_import_residual(0, torch.from_numpy(e).to(H.DEV), state)
    ctx.mc_state_export_residual(0, state, back)
    assert H.same_bits(back.cpu().numpy(), e)
    # a compress that starts from an imported residual equals the oracle started from that residual
    g = rng.standard_normal(n, dtype=np.float32)
    ocfg = O.Config(H.ALGOS[algo], ratio_ppm=10000)
    ost = e.copy()
    op, _ = O.compress(ocfg, g, ost, worker=1, it=7)
    pay = torch.zeros(ctx.payload_bytes(0), dtype=torch.uint8, device=H.DEV)
    ctx.mc_compress(0, 1, 7, [torch.from_numpy(g).to(H.DEV)], state, pay)
    ctx.mc_state_export_residual(0, state, back)
    gp = pay.cpu().numpy()
    if not H.check_payload(algo, gp, op, f"{algo} after import"):
        # the group scalar differs in its last bits (allowed: 1e-6): the oracle encodes again with the GPU's
        gh = O.header(gp)
        ost = e.copy()
        op, _ = O.compress(ocfg, g, ost, worker=1, it=7, scale_in=(gh["scale"], gh["scale2"]) if algo == "onebit" else gh["scale"])
    assert np.array_equal(gp, op) and H.same_bits(back.cpu().numpy(), ost)
    ctx.close()


def test_state_calls_on_a_stateless_algorithm_touch_nothing():
    """SignSGD keeps no state vectors: import and export are no-ops, whatever the group's size (an import used to write
    the group's n floats behind the 128-byte state)."""
    n = 50000
    ctx = B.Context("signsgd", [n], [0, 1])
    assert ctx.state_bytes(0) == 128
    buf = torch.full((128 + 4 * n + 256,), 0x5A, dtype=torch.uint8, device=H.DEV)     # the state, then memory that is not its own
    L = B.lib()
    assert L.mc_state_import_residual(ctx._h, 0, None, buf.data_ptr(), None) == B.MC_OK
    assert L.mc_state_export_residual(ctx._h, 0, buf.data_ptr(), None, None) == B.MC_OK
    torch.cuda.synchronize()
    assert bool(torch.all(buf == 0x5A))
    assert L.mc_state_import_residual(ctx._h, 0, None, None, None) == B.MC_ERR_INVALID_ARG
    ctx.close()


@pytest.mark.parametrize("algo", ["efsign", "topk", "qsgd", "signsgd"])
def test_all_groups_in_one_call(algo):
    """mc_compress_groups / mc_decompress_sum_groups are the loops over the groups: same payloads, states and sums as
    one call per group (which the other tests compare with the oracle)."""
    numel = [3000, 17, 0, 5000, 1200, 64, 7000]
    y, W = 3, 2
    bounds = B.mc_partition(numel, y)
    ctx = B.Context(algo, numel, bounds, ratio_ppm=20000, seed=5)
    ef = algo != "signsgd"
    rng = np.random.default_rng(8)
    flats = [rng.standard_normal(sum(numel)).astype(np.float32) for _ in range(W)]
    grads = [H.device_tensors(f, numel) for f in flats]
    new = lambda fn: [[torch.zeros(fn(j), dtype=torch.uint8, device=H.DEV) for j in range(y)] for _ in range(W)]
    st_a, st_b, pay_a, pay_b = new(ctx.state_bytes), new(ctx.state_bytes), new(ctx.payload_bytes), new(ctx.payload_bytes)
    for it in range(2):
        for w in range(W):
            for j in range(y):
                ctx.mc_compress(j, w, it, grads[w][bounds[j]:bounds[j + 1]], st_a[w][j] if ef else None, pay_a[w][j])
            ctx.mc_compress_groups(w, it, grads[w], st_b[w] if ef else None, pay_b[w])
    for w in range(W):
        for j in range(y):
            assert torch.equal(pay_a[w][j], pay_b[w][j]) and torch.equal(st_a[w][j], st_b[w][j]), (w, j)
    out_a, out_b = H.empty_like_list(grads[0]), H.empty_like_list(grads[0])
    for j in range(y):
        ctx.mc_decompress_sum(j, [pay_a[w][j] for w in range(W)], 0.5, out_a[bounds[j]:bounds[j + 1]])
    ctx.mc_decompress_sum_groups([pay_b[w][j] for w in range(W) for j in range(y)], W, 0.5, out_b)
    assert H.same_bits(H.gather_flat(out_a), H.gather_flat(out_b))
    assert ctx.mc_last_device_status() == B.MC_OK
    with pytest.raises(B.McError):
        ctx.mc_decompress_sum_groups([pay_b[0][0]] * (65 * y), 65, 1.0, out_b)
    ctx.close()


def test_more_address_lists_than_the_context_caches():
    """A context keeps device copies of the tensor-address lists it has seen (256 of them); 300 different lists, then the
    first ones again: every call must read the tensors it was given, also after its list's copy was replaced."""
    numel = [1500, 700, 3000]                          # three tensors, one group: chunks that straddle tensors too
    n = sum(numel)
    ctx = B.Context("fp16", numel, [0, 3], use_ef=0)
    ocfg = O.Config(H.ALGOS["fp16"], use_ef=0)
    rng = np.random.default_rng(5)
    flats = [rng.standard_normal(n).astype(np.float32) for _ in range(300)]
    lists = [H.device_tensors(f, numel) for f in flats]
    pay = torch.zeros(ctx.payload_bytes(0), dtype=torch.uint8, device=H.DEV)
    for i in list(range(300)) + [0, 1, 2, 299, 150]:
        ctx.mc_compress(0, 0, i, lists[i], None, pay)
        opay, _ = O.compress(ocfg, flats[i], None)
        assert np.array_equal(pay.cpu().numpy(), opay), i
    assert ctx.mc_last_device_status() == B.MC_OK
    ctx.close()


def test_payload_mismatch_is_reported_not_fatal():
    n = 5000
    ctx = B.Context("efsign", [n], [0, 1])
    other = B.Context("topk", [n], [0, 1])
    g = torch.randn(n, device=H.DEV)
    st = torch.zeros(ctx.state_bytes(0), dtype=torch.uint8, device=H.DEV)
    pay = torch.zeros(ctx.payload_bytes(0), dtype=torch.uint8, device=H.DEV)
    ctx.mc_compress(0, 0, 0, [g], st, pay)
    out = torch.zeros(n, device=H.DEV)
    ctx.mc_decompress_sum(0, [pay], 1.0, [out])
    assert ctx.mc_last_device_status() == B.MC_OK
    # a sparse context fed an EF-Sign payload: flagged; garbage indices are never written out of bounds
    big = torch.zeros(max(other.payload_bytes(0), ctx.payload_bytes(0)), dtype=torch.uint8, device=H.DEV)
    big[:pay.numel()] = pay
    guard = torch.full((n + 64,), 7.0, device=H.DEV)
    other.mc_decompress_sum(0, [big], 1.0, [guard[32:32 + n]])
    assert other.mc_last_device_status() == B.MC_ERR_PAYLOAD
    assert other.mc_last_device_status() == B.MC_OK            # the flag is cleared by reading it
    assert torch.all(guard[:32] == 7.0) and torch.all(guard[32 + n:] == 7.0)
    # host-side argument checks
    L = B.lib()
    assert L.mc_compress(ctx._h, 3, 0, 0, None, None, None, None) == B.MC_ERR_INVALID_ARG
    with pytest.raises(B.McError):
        ctx.mc_compress(0, 0, 0, [g], None, pay)               # use_ef = 1 needs a state
    with pytest.raises(B.McError):
        ctx.mc_decompress_sum(0, [pay] * 65, 1.0, [out])       # more than 64 payloads
    with pytest.raises(B.McError):
        ctx.mc_compress(0, 0, 0, [g], st, pay[4:])             # payload not 16-byte aligned
    ctx.close(); other.close()


def test_profile_hooks_count_launches():
    n = 100000
    ctx = B.Context("efsign", [n], [0, 1])
    g = torch.randn(n, device=H.DEV)
    st = torch.zeros(ctx.state_bytes(0), dtype=torch.uint8, device=H.DEV)
    pay = torch.zeros(ctx.payload_bytes(0), dtype=torch.uint8, device=H.DEV)
    ctx.profile_enable(True)
    for it in range(3):
        ctx.mc_compress(0, 0, it, [g], st, pay)
    prof = ctx.profile_read()
    assert prof["efsign_compress"]["launches"] == 3 and prof["scalar_finalize"]["launches"] == 3
    assert prof["efsign_compress"]["total_ms"] > 0
    assert prof["upload_ptrs"]["launches"] == 2                # address list uploaded + expanded once, then cached
    ctx.profile_reset()
    ctx.profile_enable(False)
    ctx.mc_compress(0, 0, 3, [g], st, pay)
    assert ctx.profile_read() == {}
    ctx.close()


def test_filter_margin_tightens_and_recovers_from_a_miss():
    """A static gradient under error feedback piles the values up below the threshold: the library narrows its
    candidate filter call by call.  Then the residual is dropped, the threshold falls far below the filter (a miss),
    and the calls after it must be exact again and return to the fast route."""
    n, tensors = 200000, [150000, 50000]
    ctx = B.Context("topk", tensors, [0, 2], ratio_ppm=10000, seed=4)
    ocfg = O.Config(O.TOPK, ratio_ppm=10000, seed=4)
    st = torch.zeros(ctx.state_bytes(0), dtype=torch.uint8, device=H.DEV)
    pay = torch.zeros(ctx.payload_bytes(0), dtype=torch.uint8, device=H.DEV)
    ost = O.new_state(ocfg, n)
    g = (np.random.default_rng(5).standard_normal(n, dtype=np.float32) * np.float32(0.01)).astype(np.float32)
    dev = H.device_tensors(g, tensors)
    routes = []
    for it in range(40):
        if it == 24:                      # forget the accumulated residual
            st.zero_()
            ost[:] = 0
        ctx.mc_compress(0, 0, it, dev, st, pay)
        routes.append(ctx.mc_last_select_route())
        op, _ = O.compress(ocfg, g, ost, group_off=0, worker=0, it=it)
        assert np.array_equal(pay.cpu().numpy(), op), f"call {it} (route {routes[-1]}): payload differs"
    e = torch.empty(n, dtype=torch.float32, device=H.DEV)
    ctx.mc_state_export_residual(0, st, e)
    assert H.same_bits(e.cpu().numpy(), ost)
    print("routes", routes, flush=True)
    assert B.MC_SELECT_FAST in routes[4:24] and routes[24] == B.MC_SELECT_REFILL and routes[-1] == B.MC_SELECT_FAST
    ctx.close()


@pytest.mark.parametrize("algo", ["topk", "dgc", "randk"])
def test_crowded_tiles_on_the_usual_route(algo):
    """The two kernels after the streaming pass read a tile's candidates as four heads of 64 and units of 256.  Gradients
    whose large values crowd into a few tiles (some chunks with more than 64 candidates, one tile with all 4096 of its
    elements above the threshold: more than four units) are compressed call after call, so that after the first calls the
    threshold stays inside the window of the last one; every payload and residual is compared."""
    numel = [50000, 4096 * 3 + 5, 70000, 777]
    n = sum(numel)
    rng0 = np.random.default_rng(91)
    scale = np.full(n, 1e-3, np.float32)
    scale[50000 + 100:50000 + 100 + 4096 + 900] = 1.0            # one tile and a bit: every element far above the rest
    scale[90000:90000 + 1500] = 0.3                              # crowded chunks
    scale[rng0.integers(0, n, 400)] = 0.5                        # and loners everywhere

    def grads(w, it):
        rng = np.random.default_rng([92, w, it])
        return rng.standard_normal(n, dtype=np.float32) * scale * np.float32(1.0 + 0.02 * it)
    st = H.run_parity(numel, algo, 1, 2, 7, grads, ratio_ppm=30000, dgc_momentum=0.3, seed=9)
    assert st.compress_checks == 14


def test_threshold_bin_too_full_to_list():
    """More keys share the threshold's window bin than the list between the select and the emit kernel holds (here: heavy
    ties at the threshold): that bin is resolved as a radix level instead.  Route and results are checked."""
    n, tensors = 200000, [120000, 80000]
    ctx = B.Context("topk", tensors, [0, 2], ratio_ppm=100000, seed=1)
    ocfg = O.Config(O.TOPK, ratio_ppm=100000, seed=1)
    st = torch.zeros(ctx.state_bytes(0), dtype=torch.uint8, device=H.DEV)
    pay = torch.zeros(ctx.payload_bytes(0), dtype=torch.uint8, device=H.DEV)
    ost = O.new_state(ocfg, n)
    rng = np.random.default_rng(3)
    routes = []
    for it in range(5):
        # 30 % of the elements carry the very same magnitude, which is where the 10 % threshold falls; error feedback off
        # for them (they are re-drawn each call), so the threshold key does not move
        g = (rng.standard_normal(n, dtype=np.float32) * np.float32(1e-3)).astype(np.float32)
        tie = rng.random(n) < 0.3
        g[tie] = np.where(rng.random(int(tie.sum())) < 0.5, 1.0, -1.0).astype(np.float32)
        ost[:] = 0
        st.zero_()
        ctx.mc_compress(0, 0, it, H.device_tensors(g, tensors), st, pay)
        routes.append(ctx.mc_last_select_route())
        op, _ = O.compress(ocfg, g, ost, group_off=0, worker=0, it=it)
        assert np.array_equal(pay.cpu().numpy(), op), f"call {it} (route {routes[-1]}): payload differs"
        e = torch.empty(n, dtype=torch.float32, device=H.DEV)
        ctx.mc_state_export_residual(0, st, e)
        assert H.same_bits(e.cpu().numpy(), ost), f"call {it}: residual differs"
    print("routes", routes, ctx.mc_select_stats(), flush=True)
    assert B.MC_SELECT_DENSE in routes
    ctx.close()


def test_a_barrier_that_is_not_passed_is_reported_and_nothing_hangs():
    """The rare selection routes run as one kernel whose blocks wait for each other, a bounded number of looks.  With
    the bound set to one look (from the host), the first call of a context -- which takes such a route, on four blocks
    here -- gives up at its first barrier: every kernel still ends, the status says so, and with the default bound
    restored the same call gives the oracle's payload."""
    n, tensors = 200000, [120000, 80000]
    ctx = B.Context("topk", tensors, [0, 2], ratio_ppm=10000, use_ef=0, seed=1)
    ocfg = O.Config(O.TOPK, ratio_ppm=10000, use_ef=0, seed=1)
    g = np.random.default_rng(11).standard_normal(n).astype(np.float32)
    grads = H.device_tensors(g, tensors)
    pay = torch.zeros(ctx.payload_bytes(0), dtype=torch.uint8, device=H.DEV)
    ctx.mc_set_barrier_spin_limit(1)
    ctx.mc_compress(0, 0, 0, grads, None, pay)
    assert B.lib().mc_last_device_status(ctx._h) == B.MC_ERR_DEVICE
    assert ctx.mc_last_device_status() == B.MC_OK                      # (the flag was cleared)
    ctx.mc_set_barrier_spin_limit(0)
    ctx.mc_compress(0, 0, 0, grads, None, pay)
    assert ctx.mc_last_device_status() == B.MC_OK
    op, _ = O.compress(ocfg, g, None, group_off=0, worker=0, it=0)
    assert np.array_equal(pay.cpu().numpy(), op)
    with pytest.raises(B.McError):
        B.Context("efsign", tensors, [0, 2]).mc_set_barrier_spin_limit(1)
    ctx.close()


def test_filter_margin_tightens_and_backs_off_after_a_miss():
    """The candidate filter starts a margin below the last threshold; the library halves the margin while many more than
    k elements pass it (here 20 000 values sit 0.3 % below the threshold of k = 4000), down to 0.8 %.  A threshold that
    then falls by 2 % is missed (a second streaming pass, the result as exact as ever); afterwards the margin may be
    halved one time less than it had been, for 64 calls.  Every payload is compared with the oracle."""
    n, tensors, k = 400000, [150000, 250000], 4000
    ctx = B.Context("topk", tensors, [0, 2], ratio_ppm=10000, use_ef=0, seed=1)
    ocfg = O.Config(O.TOPK, ratio_ppm=10000, use_ef=0, seed=1)
    rng = np.random.default_rng(2)
    g = (rng.standard_normal(n, dtype=np.float32) * np.float32(1e-3)).astype(np.float32)
    pos = rng.choice(n, k + 20000, replace=False)
    g[pos[:k]] = (2.0 + rng.random(k)).astype(np.float32)
    g[pos[k:]] = np.float32(1.994) - rng.random(20000).astype(np.float32) * np.float32(1e-3)
    pay = torch.zeros(ctx.payload_bytes(0), dtype=torch.uint8, device=H.DEV)
    it = [0]

    def call(grad):
        ctx.mc_compress(0, 0, it[0], H.device_tensors(grad, tensors), None, pay)
        op, _ = O.compress(ocfg, grad, None, group_off=0, worker=0, it=it[0])
        assert np.array_equal(pay.cpu().numpy(), op), f"call {it[0]}"
        it[0] += 1
        s = ctx.mc_select_stats()
        return ctx.mc_last_select_route(), s["margin_halvings"], s["margin_cap"]

    assert ctx.mc_select_stats()["margin_halvings"] == -1
    log = [call(g) for _ in range(16)]
    assert log[-1] == (B.MC_SELECT_FAST, 4, 4), log                       # after the first call's hold: four halvings
    g2 = (g * np.float32(0.98)).astype(np.float32)
    assert call(g2) == (B.MC_SELECT_REFILL, 0, 3)                          # the miss: margin back to full, capped one step lower
    log = [call(g2) for _ in range(30)]
    assert all(r == B.MC_SELECT_FAST for r, _, _ in log) and max(h for _, h, _ in log) == 3 and log[-1][1:] == (3, 3), log
    log = [call(g2) for _ in range(50)]                                    # 64 calls after the miss the cap is lifted
    assert log[-1] == (B.MC_SELECT_FAST, 4, 4), log
    assert ctx.mc_last_device_status() == B.MC_OK
    ctx.close()


@pytest.mark.parametrize("inbin", [40, 900, 3500])
def test_long_list_of_keys_in_the_threshold_bin(inbin):
    """The usual route with `inbin` different keys in the threshold's window bin (2048 consecutive keys): the emit kernel
    asks for the first sixteen entries of each of the list's 64 sublists before it knows their lengths and fetches the
    rest afterwards; 40 keys leave most sublists empty, 900 fill them unevenly around the sixteen, 3500 go far beyond."""
    n, tensors = 400000, [150000, 250000]
    k = 4000
    ctx = B.Context("topk", tensors, [0, 2], ratio_ppm=10000, use_ef=0, seed=1)
    ocfg = O.Config(O.TOPK, ratio_ppm=10000, use_ef=0, seed=1)
    assert ctx.group_k(0) == k
    pay = torch.zeros(ctx.payload_bytes(0), dtype=torch.uint8, device=H.DEV)
    rng = np.random.default_rng(inbin)
    routes, bins = [], []
    for it in range(4):
        g = (rng.standard_normal(n, dtype=np.float32) * np.float32(1e-3)).astype(np.float32)
        # k - inbin / 2 values well above 1, and `inbin` values 1 + j ulp, j < 2048 (one bin of the window holds them all
        # if it starts at a multiple of 2048 keys from the hint: two adjacent bins otherwise, which still makes long sublists)
        pos = rng.choice(n, k - inbin // 2 + inbin, replace=False)
        g[pos[:k - inbin // 2]] = (2.0 + rng.random(k - inbin // 2)).astype(np.float32) * np.where(rng.random(k - inbin // 2) < 0.5, 1, -1).astype(np.float32)
        keys = np.uint32(0x3F800000) + rng.choice(2048, inbin, replace=inbin > 2048).astype(np.uint32)
        g[pos[k - inbin // 2:]] = keys.view(np.float32) * np.where(rng.random(inbin) < 0.5, 1, -1).astype(np.float32)
        ctx.mc_compress(0, 0, it, H.device_tensors(g, tensors), None, pay)
        routes.append(ctx.mc_last_select_route())
        bins.append(ctx.mc_select_stats()["last_bin_keys"])
        op, _ = O.compress(ocfg, g, None, group_off=0, worker=0, it=it)
        assert np.array_equal(pay.cpu().numpy(), op), f"call {it} (route {routes[-1]}): payload differs"
    print("routes", routes, "keys in the bin", bins, flush=True)
    assert routes[1:] == [B.MC_SELECT_FAST] * 3 and max(bins[1:]) >= inbin // 2
    assert ctx.mc_last_device_status() == B.MC_OK
    ctx.close()


@pytest.mark.parametrize("algo", ["topk", "dgc"])
def test_selection_routes_are_all_taken_and_exact(algo):
    """The exact selection has three routes: the threshold key T falls inside the histogram window that the
    library keeps from (last T - 3/16 octave) upward over 2047 bins of 2048 keys; above it; or below its start
    (too few candidates -> second streaming pass).  Drive one (group, worker) through all three by scaling the
    gradients; the route expected follows from the oracle's thresholds; every payload and residual is compared."""
    n, tensors = 300000, [120000, 7, 179993]
    ctx = B.Context(algo, tensors, [0, 3], ratio_ppm=10000, dgc_momentum=0.0, seed=3)
    ocfg = O.Config(H.ALGOS[algo], ratio_ppm=10000, dgc_momentum=0.0, seed=3)
    st = torch.zeros(ctx.state_bytes(0), dtype=torch.uint8, device=H.DEV)
    pay = torch.zeros(ctx.payload_bytes(0), dtype=torch.uint8, device=H.DEV)
    ost = O.new_state(ocfg, n)
    k = ctx.group_k(0)
    rng = np.random.default_rng(77)
    hint, seen = 0, []
    for it, scale in enumerate([1.0, 0.3, 0.3, 64.0, 20.0, 20.0, None, 1e-3]):
        if scale is None:                 # forget the accumulated residual: the next, tiny, gradient stands alone
            st.zero_()
            ost[:] = 0
            continue
        g = (rng.standard_normal(n, dtype=np.float32) * np.float32(scale)).astype(np.float32)
        ctx.mc_compress(0, 5, it, H.device_tensors(g, tensors), st, pay)
        got = ctx.mc_last_select_route()
        op, _ = O.compress(ocfg, g, ost, group_off=0, worker=5, it=it)
        T = int((O.sparse_view(op)[1].view(np.uint32) & 0x7FFFFFFF).min())           # k-th largest key
        want = B.MC_SELECT_REFILL if T < hint else B.MC_SELECT_FAST if T - hint < 2047 * 2048 else B.MC_SELECT_ABOVE
        assert got == want, f"call {it}: route {got}, expected {want} (T {T:#x}, hint {hint:#x})"
        hint = T - (3 << 19) if T > (3 << 19) else 0
        seen.append(got)
        assert np.array_equal(pay.cpu().numpy(), op), f"call {it} (route {got}): payload differs"
        e = torch.empty(O.state_floats(ocfg, n), dtype=torch.float32, device=H.DEV)
        ctx.mc_state_export_residual(0, st, e)
        assert H.same_bits(e.cpu().numpy(), ost), f"call {it}: residual differs"
    assert set(seen) == {B.MC_SELECT_ABOVE, B.MC_SELECT_FAST, B.MC_SELECT_REFILL}, seen
    # another worker id of the same context has no hint of its own yet
    ctx.mc_compress(0, 6, 9, H.device_tensors(g, tensors), torch.zeros_like(st), pay)
    assert ctx.mc_last_select_route() == B.MC_SELECT_ABOVE
    ctx.close()
