"""Pins for the CPU oracle: what the paper and the mathematics fix, checked without a GPU.

Each pin states where it comes from.  Both oracle implementations (numpy and
plain C) go through the same pins; a last group plants typical mistakes into
copies of the rule and checks that the pins reject them.
"""

import itertools
import json
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import brace_oracle as O
from oracle import c_oracle as C


# --------------------------------------------------------------------------
# the two implementations behind one call shape: f(updates, lam, zero_sign) -> (out, sums)
# --------------------------------------------------------------------------

def _numpy_impl(G, lam, zs=0):
    r = O.brace_direct(np.asarray(G, dtype=np.float32), lam, zs)
    return r.out, r.sums


def _c_impl(G, lam, zs=0):
    out, sums, _ = C.brace_direct(np.ascontiguousarray(G, dtype=np.float32), lam, zs)
    return out, sums.astype(np.int64)


def _loops_impl(G, lam, zs=0):
    G = np.asarray(G, dtype=np.float32)
    out = np.array(O.brace_direct_loops(G.tolist(), lam, zs), dtype=np.float32)
    return out, None


IMPLS = {"numpy": _numpy_impl, "c": _c_impl, "loops": _loops_impl}


@pytest.fixture(params=sorted(IMPLS))
def impl(request):
    return IMPLS[request.param]


def _golden(golden_dir, name):
    with open(os.path.join(golden_dir, name)) as fh:
        return json.load(fh)


# --------------------------------------------------------------------------
# Eq. (1): printed definition, tie rule, appendix identity
# --------------------------------------------------------------------------

def test_derived_example_lambda2(impl, golden_dir):
    # Sec. 2.2 gradients with Sec. 3's illustration threshold; worked by hand in the fixture.
    ex = _golden(golden_dir, "brace_parameters.json")["derived_example"]
    out, sums = impl(ex["gradients"], ex["lambda"])
    assert out.tolist() == [float(v) for v in ex["output"]]
    if sums is not None:
        assert sums.tolist() == ex["sign_sums"]


def test_tie_goes_to_minus_one(impl):
    # Eq. (1): sum <= lambda -> -1, so sum == lambda is -1 and sum == lambda + 1 is +1.
    for n in (1, 2, 5, 8):
        for p in range(n + 1):
            col = np.array([1.0] * p + [-1.0] * (n - p), dtype=np.float32)[:, None]
            s = 2 * p - n
            out, _ = impl(col, float(s))
            assert out[0] == -1.0
            out, _ = impl(col, float(s - 1))
            assert out[0] == 1.0
            out, _ = impl(col, s - 0.5)
            assert out[0] == 1.0
            out, _ = impl(col, s + 0.5)
            assert out[0] == -1.0


def test_brute_force_all_sign_patterns(impl):
    # Every pattern in {-1, 0, +1}^n for n <= 5, every integer and half-integer
    # threshold in [-n-1, n+1].  Expected value from counting by hand:
    # S = P - N + zero_sign * Z, output +1 iff S > lambda.
    vals = np.array([-2.5, 0.0, 0.75], dtype=np.float32)
    for n in (1, 2, 3, 4, 5):
        pats = np.array(list(itertools.product(range(3), repeat=n)))      # (3^n, n)
        G = vals[pats].T.copy()                                           # (n, 3^n)
        P = (pats == 2).sum(1)
        N = (pats == 0).sum(1)
        Z = (pats == 1).sum(1)
        for zs in (-1, 0, 1):
            S = P - N + zs * Z
            for lam2 in range(-2 * n - 2, 2 * n + 3):
                lam = lam2 / 2.0
                out, sums = impl(G, lam, zs)
                want = np.where(2 * S > lam2, 1.0, -1.0)
                assert np.array_equal(out, want), (n, zs, lam)
                if sums is not None:
                    assert np.array_equal(sums, S)


def test_appendix_identity_two_I_minus_one(impl):
    # App. A: GAR[k] = 2 * I(sum > lambda) - 1.
    rng = np.random.default_rng(11)
    G = rng.standard_normal((9, 200)).astype(np.float32)
    for lam in (-3, 0, 2, 5):
        out, _ = impl(G, lam)
        ind = (np.sign(G).sum(0) > lam).astype(np.float64)
        assert np.array_equal(out, (2 * ind - 1).astype(np.float32))


# --------------------------------------------------------------------------
# Special cases that reduce to library routines or closed forms
# --------------------------------------------------------------------------

def test_majority_vote_special_case(impl):
    # lambda = 0, n odd, no zeros: the rule is the element-wise majority sign,
    # which is also the sign of the median of the n values (library: np.median).
    rng = np.random.default_rng(5)
    for n in (1, 3, 7, 21):
        G = rng.standard_normal((n, 501)).astype(np.float32)
        assert not (G == 0).any()
        out, _ = impl(G, 0.0)
        assert np.array_equal(out, np.sign(np.median(G, axis=0)).astype(np.float32))


def test_order_statistic_form(impl):
    # No zeros: out = +1  <=>  P > (n + lambda) / 2  <=>  at least p_min values are
    # positive, p_min = floor((n + lambda) / 2) + 1  <=>  the p_min-th largest value
    # is positive (library: np.sort).
    rng = np.random.default_rng(6)
    n = 12
    G = (rng.standard_normal((n, 400)) + 0.3).astype(np.float32)
    assert not (G == 0).any()
    desc = -np.sort(-G, axis=0)
    for lam in (-4, -1, 0, 1, 2, 5, 7.5, 10):
        p_min = int(np.floor((n + lam) / 2)) + 1
        out, _ = impl(G, lam)
        if p_min > n:
            want = -np.ones(400, dtype=np.float32)
        elif p_min <= 0:
            want = np.ones(400, dtype=np.float32)
        else:
            want = np.where(desc[p_min - 1] > 0, 1.0, -1.0).astype(np.float32)
        assert np.array_equal(out, want), lam


def test_saturating_thresholds(impl):
    # |S| <= n, so lambda >= n forces -1 everywhere and lambda < -n forces +1 everywhere.
    rng = np.random.default_rng(7)
    n = 6
    G = rng.standard_normal((n, 64)).astype(np.float32)
    G[:, 0] = 1.0
    G[:, 1] = -1.0
    for lam in (n, n + 0.5, 1e9):
        out, _ = impl(G, lam)
        assert (out == -1).all()
    for lam in (-n - 0.5, -n - 1, -1e9):
        out, _ = impl(G, lam)
        assert (out == 1).all()
    out, _ = impl(G, -n)          # S = -n is not > -n
    assert out[1] == -1 and out[0] == 1
    out, _ = impl(G, n - 1)       # only the unanimous +1 column passes
    assert out[0] == 1 and (out[1:] == -1).sum() >= 1


def test_single_client(impl):
    g = np.array([[3.0, -2.0, 0.0, -0.0, np.inf, -np.inf, np.nan, 1e-45, -1e-45]], dtype=np.float32)
    out, sums = impl(g, 0.0)
    assert out.tolist() == [1, -1, -1, -1, 1, -1, -1, 1, -1]
    if sums is not None:
        assert sums.tolist() == [1, -1, 0, 0, 1, -1, 0, 1, -1]
    out, _ = impl(g, -1.0)        # S > -1 <=> S in {0, 1}
    assert out.tolist() == [1, -1, 1, 1, 1, -1, 1, 1, -1]


def test_special_values_and_zero_sign(impl):
    # Readings for what the paper leaves open: +-0 and NaN vote zero_sign; infinities
    # and denormals keep their sign.
    col = np.array([0.0, -0.0, np.nan, np.inf, -np.inf, 1e-45, -1e-45, 2.0], dtype=np.float32)[:, None]
    for zs, s in ((0, 1), (1, 4), (-1, -2)):
        out, sums = impl(col, 0.0, zs)
        if sums is not None:
            assert sums[0] == s
        assert out[0] == (1.0 if s > 0 else -1.0)


# --------------------------------------------------------------------------
# Invariants of the rule
# --------------------------------------------------------------------------

def _mixed(rng, n, d):
    G = rng.standard_normal((n, d)).astype(np.float32)
    G[rng.random((n, d)) < 0.1] = 0.0
    G[rng.random((n, d)) < 0.02] = -0.0
    return G


def test_permutation_invariance(impl):
    rng = np.random.default_rng(21)
    G = _mixed(rng, 11, 300)
    base, _ = impl(G, 2.0)
    for _ in range(5):
        out, _ = impl(G[rng.permutation(11)], 2.0)
        assert np.array_equal(out, base)


def test_positive_scaling_invariance(impl):
    rng = np.random.default_rng(22)
    G = _mixed(rng, 8, 300)
    base, _ = impl(G, 1.0)
    a = rng.uniform(0.5, 1e6, size=(8, 1)).astype(np.float32)
    out, _ = impl(G * a, 1.0)
    assert np.array_equal(out, base)


def test_output_alphabet_and_sum_bounds(impl):
    rng = np.random.default_rng(23)
    n = 9
    G = rng.standard_normal((n, 257)).astype(np.float32)
    out, sums = impl(G, 5.0)
    assert set(np.unique(out)) <= {-1.0, 1.0}
    if sums is not None:
        assert (np.abs(sums) <= n).all()
        assert ((sums - n) % 2 == 0).all()     # no zeros: S and n have the same parity


def test_monotone_in_values_and_threshold(impl):
    rng = np.random.default_rng(24)
    n, d = 7, 200
    G = _mixed(rng, n, d)
    lam = 1.0
    base, _ = impl(G, lam)
    up = G.copy()
    i = rng.integers(0, n, size=d)
    up[i, np.arange(d)] = np.abs(up[i, np.arange(d)]) + 1.0     # raise one vote per column
    out_up, _ = impl(up, lam)
    assert (out_up >= base).all()
    prev = base
    for lam2 in (1.5, 2, 3, 6):
        cur, _ = impl(G, lam2)
        assert (cur <= prev).all()
        prev = cur


def test_bounded_influence_of_f_byzantine_rows(impl):
    # With S_b the benign sign-sum: S_b - f > lambda forces +1 and S_b + f <= lambda
    # forces -1, whatever the f Byzantine rows hold.
    rng = np.random.default_rng(25)
    n, f, d, lam = 20, 4, 400, 5.0
    benign = (rng.standard_normal((n - f, d)) + 0.8).astype(np.float32)
    S_b = np.sign(benign).sum(0)
    for trial in range(6):
        byz = rng.choice(np.array([-1e30, -1.0, -0.0, 0.0, np.nan, 1.0, 1e30, np.inf, -np.inf],
                                  dtype=np.float32), size=(f, d))
        out, _ = impl(np.vstack([benign, byz]), lam)
        assert (out[S_b - f > lam] == 1).all()
        assert (out[S_b + f <= lam] == -1).all()


# --------------------------------------------------------------------------
# Ring schedule, ownership, traffic (Sec. 2.2, Sec. 3, Table 1)
# --------------------------------------------------------------------------

def test_three_client_ring_example(golden_dir):
    ex = _golden(golden_dir, "rar_three_client_example.json")
    G = np.array(ex["gradients"], dtype=np.float32)
    res = O.ring_all_reduce(G, mode="sum", record=True)

    # step 1: Client 1 receives the third sub-vector from Client 3
    s1 = ex["share_reduce_step1"]
    hits = [m for m in res.messages if m.phase == "share_reduce" and m.step == 1
            and m.dst == s1["receiver"] - 1]
    assert len(hits) == 1
    assert hits[0].src == s1["sender"] - 1 and hits[0].chunk == s1["sub_vector"] - 1

    # ... and forwards the reduced value -2 to Client 2
    fw = ex["client1_forwards"]
    hits = [m for m in res.messages if m.phase == "share_reduce" and m.step == 2 and m.src == 0]
    assert len(hits) == 1
    assert hits[0].dst == fw["to"] - 1 and hits[0].chunk == fw["sub_vector"] - 1
    assert hits[0].payload.tolist() == [fw["value"]]

    # after n-1 steps Client 1 holds the aggregated second sub-vector, value 1
    own = ex["after_share_reduce"]
    c, vals = res.owned_after_reduce[own["client"] - 1]
    assert c == own["holds_sub_vector"] - 1 and vals.tolist() == [own["value"]]
    for c in range(3):
        assert O.chunk_owner(3, c) == (c - 1) % 3
    assert O.chunk_owner(3, own["holds_sub_vector"] - 1) == own["client"] - 1

    # every client ends with the full sum
    for b in res.buffers:
        assert b.tolist() == [22, 1, 5]

    # the compromised variant printed in Sec. 3
    G2 = G.copy()
    G2[0] = ex["attacked_gradient_client1"]
    res2 = O.ring_all_reduce(G2, mode="sum")
    for b in res2.buffers:
        assert b.tolist() == ex["attacked_aggregate"]
    assert O.rar_sum_direct(G2).tolist() == ex["attacked_aggregate"]
    assert C.rar_sum(G2).tolist() == ex["attacked_aggregate"]


@pytest.mark.parametrize("n,d", [(1, 5), (2, 2), (3, 3), (4, 10), (5, 3), (7, 23), (10, 100), (6, 0)])
def test_ring_brace_all_clients_identical_and_equal_to_definition(n, d):
    # Sec. 3 Phase IV: all clients receive the same vector; it must be Eq. (1) everywhere.
    rng = np.random.default_rng(100 + n + d)
    G = _mixed(rng, n, d) if d else np.zeros((n, 0), dtype=np.float32)
    for lam in (-1, 0, 2):
        for zs in (0, 1, -1):
            res = O.ring_all_reduce(G, mode="brace", lam=lam, zero_sign=zs)
            want = O.brace_direct(G, lam, zs)
            for b in res.buffers:
                assert np.array_equal(b, want.out)
            for i, (c, vals) in enumerate(res.owned_after_reduce):
                lo, hi = O.chunk_range(n, d, c)
                assert O.chunk_owner(n, c) == i
                assert np.array_equal(vals, want.sums[lo:hi])


def test_ring_sum_equals_direct_sum():
    rng = np.random.default_rng(3)
    G = rng.standard_normal((6, 41)).astype(np.float32)
    res = O.ring_all_reduce(G, mode="sum")
    want = O.rar_sum_direct(G)
    for b in res.buffers:
        np.testing.assert_allclose(b, want, rtol=1e-14, atol=1e-14)
    np.testing.assert_allclose(C.rar_sum(G), want, rtol=1e-14, atol=1e-14)
    np.testing.assert_allclose(C.rar_sum(G, 1.0 / 6), O.mean_direct(G), rtol=1e-14, atol=1e-14)


# --- the ring sum in the clients' own precision (Sec. 2.2 Share-Reduce) -------------------

def test_fp32_ring_reproduces_the_printed_example(golden_dir):
    # Small integers are exact in fp32: the printed steps and sums must come out unchanged.
    ex = _golden(golden_dir, "rar_three_client_example.json")
    G = np.array(ex["gradients"], dtype=np.float32)
    res = O.ring_all_reduce(G, mode="sum", record=True, dtype=np.float32)
    fw = ex["client1_forwards"]
    hits = [m for m in res.messages if m.phase == "share_reduce" and m.step == 2 and m.src == 0]
    assert hits[0].payload.dtype == np.float32 and hits[0].payload.tolist() == [fw["value"]]
    for b in res.buffers:
        assert b.dtype == np.float32 and b.tolist() == [22, 1, 5]
    G[0] = ex["attacked_gradient_client1"]
    assert O.rar_sum_ring_order(G).tolist() == ex["attacked_aggregate"]
    assert C.rar_sum_ring_f32(G).tolist() == ex["attacked_aggregate"]


def test_fp32_ring_order_is_c_then_c_plus_1():
    # Three clients holding (2^24, 1, 1) in EVERY coordinate.  In fp32 2^24 + 1 = 2^24 (tie to
    # even) and 2 + 2^24 = 2^24 + 2, so the order of the additions shows in the result:
    #   chunk 0: (2^24 + 1) + 1 = 2^24          order 0, 1, 2
    #   chunk 1: (1 + 1) + 2^24 = 2^24 + 2      order 1, 2, 0
    #   chunk 2: (1 + 2^24) + 1 = 2^24          order 2, 0, 1
    # which is the order the ring example of Sec. 2.2 fixes (Client 1 receives the third
    # sub-vector from Client 3, adds its own, forwards to Client 2).
    big = float(2 ** 24)
    G = np.array([[big] * 6, [1.0] * 6, [1.0] * 6], dtype=np.float32)
    want = [big, big, big + 2, big + 2, big, big]
    assert O.rar_sum_ring_order(G).tolist() == want
    assert C.rar_sum_ring_f32(G).tolist() == want
    res = O.ring_all_reduce(G, mode="sum", dtype=np.float32)
    for b in res.buffers:
        assert b.tolist() == want
    # the exact sum is 2^24 + 2 everywhere; the fp64 route gives it
    assert O.rar_sum_direct(G).tolist() == [big + 2] * 6
    # reversed ring direction (c, c-1, ...) or index order 0..n-1 would give other vectors
    idx_order = G[0] + G[1] + G[2]
    assert idx_order.tolist() != want


@pytest.mark.parametrize("n,d", [(1, 7), (2, 9), (3, 3), (5, 3), (7, 23), (10, 1000), (20, 1003)])
def test_fp32_ring_order_equals_the_message_by_message_ring(n, d):
    rng = np.random.default_rng(7 * n + d)
    G = (rng.standard_normal((n, d)) * 10.0 ** rng.integers(-3, 4, size=(n, 1))).astype(np.float32)
    want = O.ring_all_reduce(G, mode="sum", dtype=np.float32)
    got = O.rar_sum_ring_order(G)
    for b in want.buffers:                                  # every client ends with the same bits
        assert np.array_equal(b.view(np.uint32), got.view(np.uint32))
    assert np.array_equal(C.rar_sum_ring_f32(G).view(np.uint32), got.view(np.uint32))
    padded = np.full((n, d + 5), np.nan, dtype=np.float32)  # the C loop honours the row pitch
    padded[:, :d] = G
    assert np.array_equal(C.rar_sum_ring_f32(padded[:, :d]).view(np.uint32), got.view(np.uint32))
    for k0, k1 in ((0, d), (0, d // 2), (d // 3, d), (d // 2, d // 2 + 1)):   # column tiles
        tile = np.ascontiguousarray(G[:, k0:k1])
        assert np.array_equal(C.rar_sum_ring_f32(tile, d_total=d, k0=k0).view(np.uint32),
                              got[k0:k1].view(np.uint32))
    mean = O.mean_ring_order(G)
    assert mean.dtype == np.float32
    assert np.array_equal(C.rar_sum_ring_f32(G, mean=True).view(np.uint32), mean.view(np.uint32))
    assert np.array_equal(mean, got / np.float32(n))
    # forward error bound of recursive summation: |err| <= (n - 1) u sum|g_i| (+ higher order)
    exact = O.rar_sum_direct(G)
    bound = (n - 1) * 2.0 ** -24 * np.abs(G.astype(np.float64)).sum(axis=0) * 1.01 + 1e-45
    assert (np.abs(got.astype(np.float64) - exact) <= bound).all()


def test_fp32_ring_misses_the_float_bar_under_cancellation_and_fp64_does_not():
    # Why the library's default sum accumulates in fp64: with Byzantine rows of magnitude 200
    # next to benign values of 0.1 (workload 1), a ring of fp32 clients lands outside
    # 1e-6 + 1e-5 |sum| of the exact sum on some coordinates, while on workload 0 (no large
    # rows) it stays inside.  Both facts are properties of the arithmetic, not of a kernel.
    from paper_2501_17392_amd import synth
    for w, some_outside in ((synth.WORKLOADS[0], False), (synth.WORKLOADS[1].with_d(200_003), True)):
        G = synth.generate(w, "cpu").numpy()
        exact = O.rar_sum_direct(G)
        ring = C.rar_sum_ring_f32(G).astype(np.float64)
        outside = np.abs(ring - exact) > 1e-6 + 1e-5 * np.abs(exact)
        assert bool(outside.any()) == some_outside
        once = exact.astype(np.float32).astype(np.float64)       # fp64 sum rounded once
        assert (np.abs(once - exact) <= 1e-6 + 1e-5 * np.abs(exact)).all()


def test_fp32_ring_order_with_more_clients_than_coordinates():
    # d < n: chunks d .. n-1 are empty, chunk c < d is the single coordinate c.
    G = np.arange(1, 1 + 5 * 3, dtype=np.float32).reshape(5, 3)
    assert O.rar_sum_ring_order(G).tolist() == G.sum(axis=0).tolist()
    assert C.rar_sum_ring_f32(G).tolist() == G.sum(axis=0).tolist()


@pytest.mark.parametrize("n,d,m", [(3, 3, 32), (4, 40, 32), (10, 1000, 16), (5, 25, 8)])
def test_ring_traffic_matches_table_1(n, d, m):
    # n | d: every client sends exactly 2md(n-1)/n bits in RAR and d(n-1)(m+1)/n in BRACE.
    rng = np.random.default_rng(9)
    G = rng.standard_normal((n, d)).astype(np.float32)
    rar = O.ring_all_reduce(G, mode="sum", m_bits=m)
    brace = O.ring_all_reduce(G, mode="brace", lam=0, m_bits=m)
    assert all(Fraction(b) == O.cost_rar(m, n, d) for b in rar.bits_sent)
    assert all(Fraction(b) == O.cost_brace(m, n, d) for b in brace.bits_sent)
    assert O.cost_rar(m, n, d) == Fraction(2 * m * d * (n - 1), n)
    assert O.cost_brace(m, n, d) == Fraction(d * (n - 1) * (m + 1), n)
    assert O.cost_sc(m, n, d) == m * n * d
    assert O.cost_brace(m, n, d) < O.cost_rar(m, n, d)        # since m > 1


def test_traffic_at_headline_shape():
    # m = 32, n = 100, d = 25 M: ratio (m + 1) / (2 m) = 33 / 64.
    rar = O.cost_rar(32, 100, 25_000_000)
    brace = O.cost_brace(32, 100, 25_000_000)
    assert brace / rar == Fraction(33, 64)
    assert rar == 1_584_000_000 and brace == 816_750_000


# --------------------------------------------------------------------------
# Chunk partition (reading: balanced, contiguous, ascending)
# --------------------------------------------------------------------------

@pytest.mark.parametrize("n,d", [(1, 0), (1, 7), (3, 3), (10, 10_000), (20, 1_000_003),
                                 (50, 11_173_962), (100, 25_000_000), (64, 100_000_000),
                                 (7, 3), (5, 0)])
def test_chunk_partition_tiles_the_vector(n, d):
    prev = 0
    sizes = []
    for c in range(n):
        lo, hi = O.chunk_range(n, d, c)
        assert lo == prev and hi >= lo
        sizes.append(hi - lo)
        prev = hi
    assert prev == d
    assert max(sizes) - min(sizes) <= 1
    assert sizes == sorted(sizes, reverse=True)
    assert sum(sizes) == d


def test_chunk_partition_known_sizes():
    assert [O.chunk_range(20, 1_000_003, c)[1] - O.chunk_range(20, 1_000_003, c)[0]
            for c in range(20)] == [50_001] * 3 + [50_000] * 17
    assert O.chunk_range(100, 25_000_000, 99) == (24_750_000, 25_000_000)
    assert O.chunk_range(10, 10_000, 3) == (3000, 4000)


def test_partition_independence():
    # The rule is per coordinate, so aggregating chunk by chunk gives the same vector.
    rng = np.random.default_rng(31)
    n, d = 7, 60
    G = _mixed(rng, n, d)
    whole = O.brace_direct(G, 1.0)
    glued = np.empty(d, dtype=np.float32)
    for c in range(n):
        lo, hi, out, sums = O.brace_chunk(G, c, 1.0)
        glued[lo:hi] = out
        assert np.array_equal(sums, whole.sums[lo:hi])
    assert np.array_equal(glued, whole.out)


# --------------------------------------------------------------------------
# Packed bits, C oracle plumbing
# --------------------------------------------------------------------------

def test_packed_bits_roundtrip():
    rng = np.random.default_rng(41)
    for d in (0, 1, 7, 8, 9, 63, 64, 65, 1001):
        out = rng.choice(np.array([-1.0, 1.0], dtype=np.float32), size=d)
        bits = O.pack_bits(out)
        assert bits.shape[0] == (d + 7) // 8
        un = np.unpackbits(bits, bitorder="little")[:d]
        assert np.array_equal(un, (out > 0).astype(np.uint8))
        if d % 8:
            assert bits[-1] >> (d % 8) == 0       # padding bits are zero
    assert O.pack_bits(np.array([1, -1, -1, 1, 1, 1, 1, 1, -1, 1], dtype=np.float32)).tolist() == [0b11111001, 0b10]


def test_c_oracle_matches_numpy_oracle_on_ragged_pitch():
    rng = np.random.default_rng(42)
    n, d, ld = 13, 1003, 1100
    store = np.full((n, ld), np.nan, dtype=np.float32)
    store[:, :d] = _mixed(rng, n, d)
    view = store[:, :d]
    for lam in (-2, 0, 2, 5):
        for zs in (-1, 0, 1):
            out, sums, bits = C.brace_direct(view, lam, zs)
            want = O.brace_direct(view, lam, zs)
            assert np.array_equal(out, want.out)
            assert np.array_equal(sums, want.sums)
            assert np.array_equal(bits, want.bits)
    for nt in (1, 3):
        out, _, _ = C.brace_direct(view, 2.0, 0, nthreads=nt)
        assert np.array_equal(out, O.brace_direct(view, 2.0).out)


def test_oracle_rejects_bad_arguments():
    with pytest.raises(ValueError):
        O.chunk_range(0, 5, 0)
    with pytest.raises(ValueError):
        O.chunk_range(3, 5, 3)
    with pytest.raises(ValueError):
        O.sign_quantize(np.zeros(3), 2)
    with pytest.raises(ValueError):
        O.consensus(np.zeros(3), float("nan"))
    with pytest.raises(ValueError):
        C.brace_direct(np.zeros((2, 3), dtype=np.float32), float("inf"))


# --------------------------------------------------------------------------
# Planted mistakes: the pins above must tell a wrong rule from the right one
# --------------------------------------------------------------------------

def _mutant(kind):
    def rule(G, lam, zs=0):
        G = np.asarray(G, dtype=np.float32)
        pos, neg = (G > 0), (G < 0)
        if kind == "signbit":                 # -0.0 and -NaN counted as negative
            neg = np.signbit(G)
            pos = ~neg & (G != 0)
        s = pos.sum(0).astype(np.int64) - neg.sum(0) + zs * (~pos & ~neg).sum(0)
        if kind == "dropped_negatives":
            s = pos.sum(0).astype(np.int64)
        if kind == "ge":
            out = np.where(s >= lam, 1.0, -1.0)
        elif kind == "flipped":
            out = np.where(s > lam, -1.0, 1.0)
        elif kind == "abs":                   # symmetric agreement instead of Eq. (1)
            out = np.where(np.abs(s) > lam, 1.0, -1.0)
        elif kind == "truncated_lambda":      # int(lambda) instead of the exact comparison
            out = np.where(s > int(lam), 1.0, -1.0)
        else:
            out = np.where(s > lam, 1.0, -1.0)
        return out.astype(np.float32), s
    return rule


@pytest.mark.parametrize("kind", ["ge", "flipped", "abs", "dropped_negatives", "signbit",
                                  "truncated_lambda"])
def test_pins_reject_planted_mistakes(kind, golden_dir):
    rule = _mutant(kind)
    pins = [
        lambda: test_tie_goes_to_minus_one(rule),
        lambda: test_brute_force_all_sign_patterns(rule),
        lambda: test_majority_vote_special_case(rule),
        lambda: test_order_statistic_form(rule),
        lambda: test_single_client(rule),
        lambda: test_special_values_and_zero_sign(rule),
        lambda: test_saturating_thresholds(rule),
        lambda: test_derived_example_lambda2(rule, golden_dir),
    ]
    failed = 0
    for pin in pins:
        try:
            pin()
        except AssertionError:
            failed += 1
    assert failed >= 1, f"no pin caught the planted mistake {kind!r}"


def test_unmutated_rule_passes_the_same_pins(golden_dir):
    rule = _mutant("none")
    test_tie_goes_to_minus_one(rule)
    test_brute_force_all_sign_patterns(rule)
    test_majority_vote_special_case(rule)
    test_order_statistic_form(rule)
    test_single_client(rule)
    test_special_values_and_zero_sign(rule)
    test_saturating_thresholds(rule)
    test_derived_example_lambda2(rule, golden_dir)


# --------------------------------------------------------------------------
# Model update (Sec. 2.1; App. A update rule w <- w - eta * (2 I - 1))
# --------------------------------------------------------------------------

def test_model_update_moves_every_coordinate_by_eta():
    rng = np.random.default_rng(51)
    n, d, eta, lam = 9, 300, 0.125, 2.0
    G = _mixed(rng, n, d)
    w = rng.standard_normal(d)
    agg = O.brace_direct(G, lam).out
    new = O.model_update(w, agg, eta)
    ind = (np.sign(G).sum(0) > lam)                    # the indicator I of App. A
    assert np.array_equal(new, w - eta * (2.0 * ind - 1.0))
    assert np.allclose(np.abs(new - w), eta, rtol=0, atol=1e-15)
    assert (new[ind] < w[ind]).all() and (new[~ind] > w[~ind]).all()
    # Mean rule plugged into the same update (Sec. 2.1)
    assert np.allclose(O.model_update(w, O.mean_direct(G), eta), w - eta * G.astype(np.float64).mean(0))


# --------------------------------------------------------------------------
# Quantise-once form (Phase I kept as bit planes)
# --------------------------------------------------------------------------

@pytest.mark.parametrize("n,d", [(1, 1), (3, 31), (5, 32), (4, 33), (9, 64), (7, 1000), (20, 4097)])
def test_planes_route_equals_definition(n, d):
    rng = np.random.default_rng(n * 100 + d)
    G = _mixed(rng, n, d)
    G[rng.random((n, d)) < 0.03] = np.nan
    planes = O.sign_planes(G)
    assert planes.shape == (n, O.packed_row_words(d)) and planes.dtype == np.uint32
    assert O.packed_row_words(d) % 4 == 0
    assert not (planes[:, 0::2] & planes[:, 1::2]).any()          # never both signs
    # the planes are exactly "x > 0" and "x < 0", bit b of word j <-> coordinate 32 j + b
    for i in range(n):
        for k in rng.integers(0, d, size=min(d, 50)):
            p = (int(planes[i, 2 * (k // 32)]) >> (k % 32)) & 1
            m = (int(planes[i, 2 * (k // 32) + 1]) >> (k % 32)) & 1
            assert p == int(G[i, k] > 0) and m == int(G[i, k] < 0)
    if d % 32:
        assert (planes[:, 2 * (d // 32)] >> (d % 32) == 0).all()   # padding bits are zero
    for lam in (-1, 0, 2):
        for zs in (-1, 0, 1):
            a = O.brace_from_planes(planes, d, lam, zs)
            b = O.brace_direct(G, lam, zs)
            assert np.array_equal(a.out, b.out) and np.array_equal(a.sums, b.sums)
            assert np.array_equal(a.bits, b.bits)


# --------------------------------------------------------------------------
# signSGD majority vote over the same phases (Sec. 5.2)
# --------------------------------------------------------------------------

def test_majority_rule_relation_to_eq_1():
    rng = np.random.default_rng(61)
    for n in (4, 7, 10):
        G = _mixed(rng, n, 400)
        maj = O.signsgd_majority(G)
        S = O.brace_direct(G, 0.0).sums
        assert set(np.unique(maj)) <= {-1.0, 0.0, 1.0}
        assert np.array_equal(maj == 0, S == 0)
        brace0 = O.brace_direct(G, 0.0).out          # lambda = 0: ties go to -1
        assert np.array_equal(maj[S != 0], brace0[S != 0])
        assert (brace0[S == 0] == -1).all()
    G = rng.standard_normal((9, 300)).astype(np.float32)      # odd n, no zeros: median sign
    assert np.array_equal(O.signsgd_majority(G), np.sign(np.median(G, axis=0)).astype(np.float32))


# --------------------------------------------------------------------------
# One-bit form of Phase I (every coordinate votes: zero_sign = +1 or -1)
# --------------------------------------------------------------------------

@pytest.mark.parametrize("zero_sign", [1, -1])
def test_one_bit_votes_reproduce_the_definition(zero_sign):
    rng = np.random.default_rng(5 + zero_sign)
    for n, d in ((1, 1), (3, 31), (4, 32), (5, 33), (7, 130), (9, 1000)):
        g = rng.standard_normal((n, d)).astype(np.float32)
        g[rng.random((n, d)) < 0.2] = 0.0
        g[rng.random((n, d)) < 0.1] = -0.0
        g[rng.random((n, d)) < 0.05] = np.nan
        plane = O.vote_plane(g, zero_sign)
        assert plane.shape == (n, O.vote_plane_row_words(d)) and plane.shape[1] % 4 == 0
        # bit by bit against the quantised votes, padding zero
        for i in range(n):
            for k in range(d):
                bit = (int(plane[i, k // 32]) >> (k % 32)) & 1
                assert bit == int(O.sign_quantize(g[i:i + 1, k:k + 1], zero_sign)[0, 0] > 0)
        unpacked = np.unpackbits(plane.view(np.uint8).reshape(n, -1), axis=1, bitorder="little")
        assert not unpacked[:, d:].any()
        for lam in (-n - 1, -1, 0, 0.5, 1, 2, n):
            got = O.brace_from_vote_plane(plane, d, lam)
            want = O.brace_direct(g, lam, zero_sign)
            assert np.array_equal(got.out, want.out)
            assert np.array_equal(got.sums, want.sums)
            assert np.array_equal(got.bits, want.bits)


def test_one_bit_form_refuses_abstaining_zeros():
    with pytest.raises(ValueError):
        O.vote_plane(np.zeros((2, 4), dtype=np.float32), 0)
