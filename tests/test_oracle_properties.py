"""Property tests of the CPU oracle (hypothesis): the invariants of Eq. (1) on arbitrary small
inputs, and agreement of the three statements of the rule (vectorised, plain C, Python loops,
ring simulation, bit planes)."""

import numpy as np
from hypothesis import given, settings, strategies as st
from hypothesis.extra import numpy as hnp

from oracle import brace_oracle as O
from oracle import c_oracle as C

values = st.sampled_from([-np.inf, -3.5, -1.0, -1e-45, -0.0, 0.0, 1e-45, 0.25, 2.0, np.inf, np.nan])
matrices = st.integers(1, 7).flatmap(
    lambda n: st.integers(1, 40).flatmap(
        lambda d: hnp.arrays(np.float32, (n, d), elements=values.map(np.float32))))
lams = st.one_of(st.integers(-9, 9).map(float), st.floats(-9, 9, allow_nan=False))
zero_signs = st.sampled_from([-1, 0, 1])


@settings(max_examples=150, deadline=None, derandomize=True)
@given(matrices, lams, zero_signs)
def test_all_statements_of_the_rule_agree(G, lam, zs):
    a = O.brace_direct(G, lam, zs)
    assert a.out.tolist() == O.brace_direct_loops(G.tolist(), lam, zs)
    c_out, c_sums, c_bits = C.brace_direct(np.ascontiguousarray(G), lam, zs)
    assert np.array_equal(c_out, a.out) and np.array_equal(c_sums, a.sums) and np.array_equal(c_bits, a.bits)
    ring = O.ring_all_reduce(G, mode="brace", lam=lam, zero_sign=zs)
    assert all(np.array_equal(b, a.out) for b in ring.buffers)
    p = O.brace_from_planes(O.sign_planes(G), G.shape[1], lam, zs)
    assert np.array_equal(p.out, a.out) and np.array_equal(p.sums, a.sums)


@settings(max_examples=100, deadline=None, derandomize=True)
@given(matrices, lams, zero_signs, st.randoms(use_true_random=False))
def test_invariants(G, lam, zs, rnd):
    n, d = G.shape
    base = O.brace_direct(G, lam, zs)
    assert set(np.unique(base.out)) <= {-1.0, 1.0}
    assert (np.abs(base.sums) <= n).all()
    perm = list(range(n))
    rnd.shuffle(perm)
    assert np.array_equal(O.brace_direct(G[perm], lam, zs).out, base.out)          # client order
    scale = np.array([[rnd.choice([1.0, 2.0, 8.0])] for _ in range(n)], dtype=np.float32)
    finite = np.where(np.isfinite(G), G, np.float32(1.0) * np.sign(np.nan_to_num(G)))
    assert np.array_equal(O.brace_direct(finite * scale, lam, zs).sums,
                          O.brace_direct(finite, lam, zs).sums)                    # positive scaling (no underflow)
    assert (O.brace_direct(G, lam + 1.0, zs).out <= base.out).all()                # monotone in lambda
    glued = np.concatenate([O.brace_chunk(G, c, lam, zs)[2] for c in range(n)])    # any partition
    assert np.array_equal(glued, base.out)
    assert np.array_equal(np.unpackbits(base.bits, bitorder="little")[:d], (base.out > 0).astype(np.uint8))
