"""Seeded random sweep over shapes, alignments, chunk runs, optional outputs and launch tunings:
every entry point of the C ABI against the CPU oracle on the same bytes.

The fixed cases of the other GPU test files pin the corners; this file walks the space between
them (ragged sizes, every base / pitch phase, forced tile shapes on inputs they were not chosen
for) so that a planning mistake in the host logic shows as a mismatch here.
"""

import numpy as np
import pytest
import torch

from oracle import brace_oracle as O
from paper_2501_17392_amd import binding as B

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
RTOL, ATOL = 1e-5, 1e-6
GUARD = 64              # elements kept around every output and checked untouched


@pytest.fixture(scope="module", autouse=True)
def _gpu_and_library():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    B.lib()
    B.brace_reset_tuning()
    yield
    B.brace_reset_tuning()


def random_shape(rng):
    n = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 9, 16, 17, 31, 40]))
    kind = rng.integers(0, 4)
    if kind == 0:
        d = int(rng.integers(1, 300))
    elif kind == 1:
        d = int(rng.integers(300, 20_000))
    elif kind == 2:
        d = int(rng.choice([1024, 2048, 4096, 8192, 65_536])) + int(rng.integers(-3, 4))
    else:
        d = int(rng.integers(20_000, 400_000 // max(1, n // 8)))
    ld = d + int(rng.choice([0, 0, 1, 2, 3, 4, 7, 8]))
    offset = int(rng.integers(0, 4))
    return n, d, ld, offset


def random_tuning(rng):
    return dict(vec=int(rng.choice([0, 0, 1, 2, 4])), cols=int(rng.choice([0, 0, 1, 2, 4, 8])),
                unroll=int(rng.choice([0, 0, 2, 4, 8])), nontemporal=int(rng.integers(0, 2)),
                pipeline=int(rng.integers(0, 2)), split_writes=int(rng.integers(0, 3)),
                rowsplit=int(rng.integers(0, 3)), stage_writes=int(rng.integers(0, 3)))


def device_matrix(g, ld, offset):
    n, d = g.shape
    store = torch.full((n * ld + offset + 8,), float("nan"), device=DEV, dtype=torch.float32)
    view = store[offset: offset + n * ld].view(n, ld)[:, :d]
    view.copy_(torch.from_numpy(g))
    return view


def guarded(d, fill, dtype, offset=0):
    """A length-d view inside a larger buffer; returns (whole, view)."""
    whole = torch.full((d + 2 * GUARD + offset,), fill, device=DEV, dtype=dtype)
    return whole, whole[GUARD + offset: GUARD + offset + d]


def untouched(whole, d, fill, offset=0):
    h = whole.cpu().numpy()
    return (h[: GUARD + offset] == fill).all() and (h[GUARD + offset + d:] == fill).all()


def votes_matrix(rng, n, d):
    g = rng.standard_normal((n, d)).astype(np.float32)
    r = rng.random((n, d))
    g[r < 0.08] = 0.0
    g[(r >= 0.08) & (r < 0.11)] = -0.0
    g[(r >= 0.11) & (r < 0.13)] = np.nan
    g[(r >= 0.13) & (r < 0.14)] = np.inf
    g[(r >= 0.14) & (r < 0.15)] = -np.inf
    g[(r >= 0.15) & (r < 0.17)] = -1e-45
    return g


def chunk_run(rng, n, d):
    """A random run of ring chunks and the coordinate range it covers."""
    a = int(rng.integers(0, n))
    b = int(rng.integers(a + 1, n + 1))
    return a, b, O.chunk_range(n, d, a)[0], O.chunk_range(n, d, b - 1)[1]


@pytest.mark.parametrize("seed", range(200))
def test_vote_random_case(seed):
    rng = np.random.default_rng(1000 + seed)
    n, d, ld, offset = random_shape(rng)
    g = votes_matrix(rng, n, d)
    upd = device_matrix(g, ld, offset)
    lam = float(rng.choice([-n - 1, -1, 0, 0.5, 1, 2, 5, n // 2, n]))
    zs = int(rng.integers(-1, 2))
    tuning = random_tuning(rng)
    want = O.brace_direct(g, lam, zs)
    want_bits = bool(rng.integers(0, 2))
    want_sums = bool(rng.integers(0, 2))
    out_off = int(rng.choice([0, 0, 1, 2, 4]))
    whole_out, out = guarded(d, 7.0, torch.float32, out_off)
    bits = torch.full(((d + 31) // 32,), -1, device=DEV, dtype=torch.int32) if want_bits else None
    whole_sums, sums = guarded(d, 12345, torch.int16) if want_sums else (None, None)
    mode = int(rng.integers(0, 3))          # whole vector / one run of chunks / every chunk in turn
    tag = dict(seed=seed, n=n, d=d, ld=ld, offset=offset, lam=lam, zs=zs, mode=mode, **tuning)
    print(tag, flush=True)
    try:
        B.brace_set_tuning(**tuning)
        if mode == 0:
            B.brace_aggregate(upd, 0, lam, zs, out=out, out_bits=bits, sums=sums)
            lo, hi = 0, d
        elif mode == 1:
            a, b, lo, hi = chunk_run(rng, n, d)
            if want_bits:
                bits.zero_()        # words shared with chunks outside the run keep their other bits
            B.brace_aggregate_chunks(upd, 0, a, b, lam, zs, out=out, out_bits=bits, sums=sums)
        else:
            if want_bits:
                bits.zero_()
            for c in rng.permutation(n):
                B.brace_aggregate_chunk(upd, 0, int(c), lam, zs, out=out, out_bits=bits, sums=sums)
            lo, hi = 0, d
    finally:
        B.brace_reset_tuning()
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.array_equal(got[lo:hi], want.out[lo:hi]), tag
    assert (got[:lo] == 7.0).all() and (got[hi:] == 7.0).all(), tag
    assert untouched(whole_out, d, 7.0, out_off), tag
    if want_sums:
        s = sums.cpu().numpy()
        assert np.array_equal(s[lo:hi].astype(np.int64), want.sums[lo:hi]), tag
        assert (s[:lo] == 12345).all() and (s[hi:] == 12345).all(), tag
        assert untouched(whole_sums, d, 12345), tag
    if want_bits:
        unpacked = np.unpackbits(bits.cpu().numpy().view(np.uint8), bitorder="little")
        assert np.array_equal(unpacked[lo:hi], (want.out[lo:hi] > 0).astype(np.uint8)), tag
        if mode != 0:
            assert not unpacked[:lo].any() and not unpacked[hi:].any(), tag
        else:
            assert not unpacked[d:].any(), tag


@pytest.mark.parametrize("seed", range(80))
def test_sum_mean_random_case(seed):
    rng = np.random.default_rng(2000 + seed)
    n, d, ld, offset = random_shape(rng)
    g = (rng.standard_normal((n, d)) * 10.0 ** rng.integers(-3, 4, size=(n, 1))).astype(np.float32)
    g[rng.random((n, d)) < 0.05] = 0.0
    upd = device_matrix(g, ld, offset)
    mean = bool(rng.integers(0, 2))
    tuning = random_tuning(rng)
    out_off = int(rng.choice([0, 0, 1, 2, 4]))
    whole, out = guarded(d, 7.0, torch.float32, out_off)
    chunk = int(rng.integers(0, n)) if rng.integers(0, 2) else None
    lo, hi = (0, d) if chunk is None else O.chunk_range(n, d, chunk)
    tag = dict(seed=seed, n=n, d=d, ld=ld, offset=offset, mean=mean, chunk=chunk, **tuning)
    print(tag, flush=True)
    try:
        B.brace_set_tuning(**tuning)
        B.brace_rar_aggregate(upd, out, mean=mean, chunk=chunk)
    finally:
        B.brace_reset_tuning()
    torch.cuda.synchronize()
    want = O.mean_direct(g) if mean else O.rar_sum_direct(g)
    got = out.cpu().numpy()
    assert np.all(np.abs(got[lo:hi].astype(np.float64) - want[lo:hi])
                  <= ATOL + RTOL * np.abs(want[lo:hi])), tag
    assert (got[:lo] == 7.0).all() and (got[hi:] == 7.0).all(), tag
    assert untouched(whole, d, 7.0, out_off), tag


@pytest.mark.parametrize("seed", range(60))
def test_ring_order_sum_random_case(seed):
    """order = 1: bit-exact against the oracle's fp32 ring, whole vector or one chunk, any tuning."""
    rng = np.random.default_rng(2500 + seed)
    n, d, ld, offset = random_shape(rng)
    g = (rng.standard_normal((n, d)) * 10.0 ** rng.integers(-3, 4, size=(n, 1))).astype(np.float32)
    g[rng.random((n, d)) < 0.05] = 0.0
    upd = device_matrix(g, ld, offset)
    mean = bool(rng.integers(0, 2))
    tuning = random_tuning(rng)
    out_off = int(rng.choice([0, 0, 1, 2, 4]))
    whole, out = guarded(d, 7.0, torch.float32, out_off)
    chunk = int(rng.integers(0, n)) if rng.integers(0, 2) else None
    lo, hi = (0, d) if chunk is None else O.chunk_range(n, d, chunk)
    tag = dict(seed=seed, n=n, d=d, ld=ld, offset=offset, mean=mean, chunk=chunk, **tuning)
    print(tag, flush=True)
    try:
        B.brace_set_tuning(**tuning)
        B.brace_rar_aggregate(upd, out, mean=mean, chunk=chunk, order=1)
    finally:
        B.brace_reset_tuning()
    torch.cuda.synchronize()
    want = O.mean_ring_order(g) if mean else O.rar_sum_ring_order(g)
    got = out.cpu().numpy()
    assert np.array_equal(got[lo:hi].view(np.uint32), want[lo:hi].view(np.uint32)), tag
    assert (got[:lo] == 7.0).all() and (got[hi:] == 7.0).all(), tag
    assert untouched(whole, d, 7.0, out_off), tag


@pytest.mark.parametrize("seed", range(40))
def test_noalloc_update_random_case(seed):
    """The allocation-free fused update against the oracle and, bit for bit, against
    brace_aggregate_update with a bit array, under any tuning."""
    rng = np.random.default_rng(3500 + seed)
    n, d, ld, offset = random_shape(rng)
    g = votes_matrix(rng, n, d)
    upd = device_matrix(g, ld, offset)
    lam = float(rng.choice([-1, 0, 1, 2, 5]))
    eta = float(rng.choice([1e-3, 0.01, 0.25, 0.5]))
    zs = int(rng.choice([0, 1, -1]))
    tuning = random_tuning(rng)
    w0 = rng.standard_normal(d).astype(np.float32)
    w_off = int(rng.choice([0, 0, 1, 2, 4]))
    whole, w = guarded(d, 5.0, torch.float32, w_off)
    w.copy_(torch.from_numpy(w0))
    ref = torch.from_numpy(w0).to(DEV)
    bits = torch.zeros(((d + 31) // 32,), device=DEV, dtype=torch.int32)
    tag = dict(seed=seed, n=n, d=d, ld=ld, offset=offset, lam=lam, eta=eta, zs=zs, **tuning)
    print(tag, flush=True)
    try:
        B.brace_set_tuning(**tuning)
        B.brace_aggregate_update_noalloc(upd, 0, w, eta, lam, zs)
        B.brace_aggregate_update(upd, 0, ref, eta, lam, zs, out_bits=bits)
    finally:
        B.brace_reset_tuning()
    torch.cuda.synchronize()
    agg = O.brace_direct(g, lam, zs).out
    want = O.model_update(w0, agg, np.float32(eta))
    got = w.cpu().numpy()
    diff = np.abs(got.astype(np.float64) - want)
    assert np.all(diff <= np.spacing(np.abs(want).astype(np.float32)).astype(np.float64)), tag
    assert np.array_equal(got, ref.cpu().numpy()), tag
    assert untouched(whole, d, 5.0, w_off), tag


@pytest.mark.parametrize("seed", range(80))
def test_update_random_case(seed):
    rng = np.random.default_rng(3000 + seed)
    n, d, ld, offset = random_shape(rng)
    g = votes_matrix(rng, n, d)
    upd = device_matrix(g, ld, offset)
    lam = float(rng.choice([-1, 0, 1, 2, 5]))
    eta = float(rng.choice([1e-3, 0.01, 0.25, 0.5]))
    tuning = random_tuning(rng)
    w0 = rng.standard_normal(d).astype(np.float32)
    w_off = int(rng.choice([0, 0, 1, 2, 4]))
    whole, w = guarded(d, 5.0, torch.float32, w_off)
    w.copy_(torch.from_numpy(w0))
    with_bits = bool(rng.integers(0, 2))
    bits = torch.zeros(((d + 31) // 32,), device=DEV, dtype=torch.int32) if with_bits else None
    chunk = int(rng.integers(0, n)) if rng.integers(0, 2) else None
    lo, hi = (0, d) if chunk is None else O.chunk_range(n, d, chunk)
    tag = dict(seed=seed, n=n, d=d, ld=ld, offset=offset, lam=lam, eta=eta, chunk=chunk,
               with_bits=with_bits, **tuning)
    print(tag, flush=True)
    try:
        B.brace_set_tuning(**tuning)
        B.brace_aggregate_update(upd, 0, w, eta, lam, out_bits=bits, chunk=chunk)
    finally:
        B.brace_reset_tuning()
    torch.cuda.synchronize()
    agg = O.brace_direct(g, lam).out
    want = O.model_update(w0, agg, np.float32(eta))
    got = w.cpu().numpy()
    diff = np.abs(got[lo:hi].astype(np.float64) - want[lo:hi])
    assert np.all(diff <= ATOL + RTOL * np.abs(want[lo:hi])), tag
    assert np.all(diff <= np.spacing(np.abs(want[lo:hi]).astype(np.float32)).astype(np.float64)), tag
    assert np.array_equal(got[:lo], w0[:lo]) and np.array_equal(got[hi:], w0[hi:]), tag
    assert untouched(whole, d, 5.0, w_off), tag
    if with_bits:
        unpacked = np.unpackbits(bits.cpu().numpy().view(np.uint8), bitorder="little")
        assert np.array_equal(unpacked[lo:hi], (agg[lo:hi] > 0).astype(np.uint8)), tag
        assert not unpacked[:lo].any() and not unpacked[hi:].any(), tag


@pytest.mark.parametrize("seed", range(60))
def test_planes_random_case(seed):
    rng = np.random.default_rng(4000 + seed)
    n, d, ld, offset = random_shape(rng)
    if seed % 5 == 0:
        d += 600_000                        # rows longer than one burst of the staged kernel
    g = votes_matrix(rng, n, d)
    upd = device_matrix(g, max(ld, d), offset)
    words = O.packed_row_words(d)
    pitch = words + 4 * int(rng.integers(0, 3))
    store = torch.full((n, pitch), -1, device=DEV, dtype=torch.int32)
    signs = store[:, :words]
    lam = float(rng.choice([-1, 0, 0.5, 1, 2, 5, n]))
    zs = int(rng.integers(-1, 2))
    stage = int(rng.integers(0, 3))
    tag = dict(seed=seed, n=n, d=d, ld=ld, offset=offset, pitch=pitch, lam=lam, zs=zs, stage=stage)
    print(tag, flush=True)
    try:
        B.brace_set_tuning(stage_writes=stage)
        B.brace_quantize(upd, signs)
    finally:
        B.brace_reset_tuning()
    whole, out = guarded(d, 7.0, torch.float32)
    bits = torch.full(((d + 31) // 32,), -1, device=DEV, dtype=torch.int32)
    B.brace_vote_packed(signs, d, 0, lam, zs, out=out, out_bits=bits)
    # a random run of chunks into buffers of its own
    a, b, lo, hi = chunk_run(rng, n, d)
    whole_c, out_c = guarded(d, 9.0, torch.float32)
    bits_c = torch.zeros((d + 31) // 32, device=DEV, dtype=torch.int32) if rng.integers(0, 2) else None
    B.brace_vote_packed_chunks(signs, d, 0, a, b, lam, zs, out=out_c, out_bits=bits_c)
    torch.cuda.synchronize()
    host = store.cpu().numpy()
    assert np.array_equal(host[:, :words].view(np.uint32), O.sign_planes(g)), tag
    assert (host[:, words:] == -1).all(), tag
    want = O.brace_direct(g, lam, zs)
    assert np.array_equal(out.cpu().numpy(), want.out), tag
    assert untouched(whole, d, 7.0), tag
    unpacked = np.unpackbits(bits.cpu().numpy().view(np.uint8), bitorder="little")
    assert np.array_equal(unpacked[:d], (want.out > 0).astype(np.uint8)), tag
    assert not unpacked[d:].any(), tag
    got_c = out_c.cpu().numpy()
    assert np.array_equal(got_c[lo:hi], want.out[lo:hi]), (tag, a, b)
    assert (got_c[:lo] == 9.0).all() and (got_c[hi:] == 9.0).all(), (tag, a, b)
    assert untouched(whole_c, d, 9.0), (tag, a, b)
    if bits_c is not None:
        unpacked_c = np.unpackbits(bits_c.cpu().numpy().view(np.uint8), bitorder="little")
        assert np.array_equal(unpacked_c[lo:hi], (want.out[lo:hi] > 0).astype(np.uint8)), (tag, a, b)
        assert not unpacked_c[:lo].any() and not unpacked_c[hi:].any(), (tag, a, b)
    if zs != 0:
        # every coordinate votes: the one-bit form must give the same vector
        vwords = O.vote_plane_row_words(d)
        vstore = torch.full((n, vwords + 4), -1, device=DEV, dtype=torch.int32)
        votes = vstore[:, :vwords]
        try:
            B.brace_set_tuning(stage_writes=stage)
            B.brace_quantize_1bit(upd, zs, votes)
        finally:
            B.brace_reset_tuning()
        whole_v, out_v = guarded(d, 5.0, torch.float32)
        B.brace_vote_1bit(votes, d, 0, lam, out=out_v)
        torch.cuda.synchronize()
        hv = vstore.cpu().numpy()
        assert np.array_equal(hv[:, :vwords].view(np.uint32), O.vote_plane(g, zs)), tag
        assert (hv[:, vwords:] == -1).all(), tag
        assert np.array_equal(out_v.cpu().numpy(), want.out), tag
        assert untouched(whole_v, d, 5.0), tag
    # receive side of Share-Only from those bits
    whole2, out2 = guarded(d, 3.0, torch.float32, 1)
    B.brace_expand_bits(bits, d, out2)
    torch.cuda.synchronize()
    assert np.array_equal(out2.cpu().numpy(), want.out), tag
    assert untouched(whole2, d, 3.0, 1), tag
