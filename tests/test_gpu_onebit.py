"""GPU parity for the one-bit form of the quantise-once route (every coordinate votes:
zero_sign = +1 or -1): brace_quantize_1bit against the oracle's vote plane and brace_vote_1bit
against the definition on the floats, bit for bit."""

import numpy as np
import pytest
import torch

from oracle import brace_oracle as O
from oracle import c_oracle as C
from paper_2501_17392_amd import binding as B
from paper_2501_17392_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module", autouse=True)
def _gpu_and_library():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    B.lib()
    B.brace_reset_tuning()
    yield
    B.brace_reset_tuning()


def special(n, d, seed):
    rng = np.random.default_rng(seed)
    g = rng.standard_normal((n, d)).astype(np.float32)
    r = rng.random((n, d))
    g[r < 0.10] = 0.0
    g[(r >= 0.10) & (r < 0.13)] = -0.0
    g[(r >= 0.13) & (r < 0.15)] = np.nan
    g[(r >= 0.15) & (r < 0.16)] = np.inf
    g[(r >= 0.16) & (r < 0.17)] = -np.inf
    g[(r >= 0.17) & (r < 0.19)] = 1e-45
    g[(r >= 0.19) & (r < 0.21)] = -1e-45
    return g


def to_device(g, ld=None, offset=0):
    n, d = g.shape
    ld = d if ld is None else ld
    store = torch.full((n * ld + offset + 8,), float("nan"), device=DEV, dtype=torch.float32)
    view = store[offset: offset + n * ld].view(n, ld)[:, :d]
    view.copy_(torch.from_numpy(g))
    return view


@pytest.mark.parametrize("n,d,ld,offset,extra", [
    (1, 1, None, 0, 0), (2, 31, None, 0, 0), (3, 32, None, 0, 0), (3, 33, None, 0, 0), (4, 127, None, 0, 0),
    (4, 128, None, 0, 0), (4, 129, None, 0, 0), (5, 1000, None, 0, 0), (3, 4095, None, 0, 0),
    (3, 4096, None, 0, 0), (3, 4097, None, 0, 0), (7, 12_345, None, 1, 4), (6, 20_000, 20_003, 2, 8),
    (10, 70_001, None, 0, 0),
    # rows longer than one 256-span burst (1,048,576 coordinates), ragged last burst and span
    (3, 1_048_576, None, 0, 0), (2, 1_048_577, None, 3, 4), (3, 2_200_003, 2_200_005, 1, 8),
    # rows of whole 16-byte vectors (the 4-dword burst kernel when bursts are forced): ragged last
    # span, last burst of one span, exactly one burst of 288 spans and one span more, padded pitch
    (2, 4, None, 0, 0), (3, 4100, None, 0, 0), (5, 12_344, 12_348, 0, 4), (2, 1_179_648, None, 0, 0),
    (2, 1_179_652, None, 4, 0), (3, 2_400_004, 2_400_008, 8, 8)])
@pytest.mark.parametrize("stage", [0, 1, 2], ids=["auto", "per-span-stores", "bursts"])
@pytest.mark.parametrize("zs", [1, -1])
def test_one_bit_quantize_matches_oracle(n, d, ld, offset, extra, stage, zs):
    g = special(n, d, seed=n * 11 + d)
    upd = to_device(g, ld, offset)
    words = B.brace_1bit_row_words(d)
    assert words == O.vote_plane_row_words(d)
    store = torch.full((n, words + extra), -1, device=DEV, dtype=torch.int32)
    votes = store[:, :words]
    B.brace_set_tuning(stage_writes=stage)
    try:
        B.brace_quantize_1bit(upd, zs, votes)
    finally:
        B.brace_reset_tuning()
    torch.cuda.synchronize()
    host = store.cpu().numpy()
    assert np.array_equal(host[:, :words].view(np.uint32), O.vote_plane(g, zs)), (n, d, stage, zs)
    assert (host[:, words:] == -1).all()


@pytest.mark.parametrize("n", [1, 2, 3, 7, 8, 9, 15, 16, 17, 100, 255, 256, 300, 1000])
def test_one_bit_vote_for_every_client_count(n):
    d = 1500
    g = special(n, d, seed=n)
    for zs in (1, -1):
        plane = O.vote_plane(g, zs)
        votes = torch.from_numpy(plane.view(np.int32).copy()).to(DEV)
        for lam in sorted({-n - 1.0, -1.0, 0.0, 0.5, 1.0, 5.0, n // 2 + 0.0, n - 1.0, float(n)}):
            want = O.brace_direct(g, lam, zs)
            assert np.array_equal(O.brace_from_vote_plane(plane, d, lam).out, want.out)
            out = torch.full((d,), 7.0, device=DEV, dtype=torch.float32)
            bits = torch.full(((d + 31) // 32,), -1, device=DEV, dtype=torch.int32)
            B.brace_vote_1bit(votes, d, 0, lam, out=out, out_bits=bits)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy(), want.out), (n, zs, lam)
            unpacked = np.unpackbits(bits.cpu().numpy().view(np.uint8), bitorder="little")
            assert np.array_equal(unpacked[:d], (want.out > 0).astype(np.uint8)), (n, zs, lam)
            assert not unpacked[d:].any()


@pytest.mark.parametrize("d", [1, 31, 32, 33, 127, 128, 129, 1023, 1024, 1025, 2048 + 77, 40_000, 100_003])
def test_one_bit_vote_output_variants(d):
    n, lam, zs = 11, 1.0, -1
    g = special(n, d, seed=d)
    upd = to_device(g)
    votes = torch.empty(n, B.brace_1bit_row_words(d), device=DEV, dtype=torch.int32)
    B.brace_quantize_1bit(upd, zs, votes)
    want = O.brace_direct(g, lam, zs)
    guard = torch.full((d + 128,), 7.0, device=DEV, dtype=torch.float32)
    out = guard[64: 64 + d]
    B.brace_vote_1bit(votes, d, 0, lam, out=out)                 # floats only (words parked in out)
    torch.cuda.synchronize()
    h = guard.cpu().numpy()
    assert np.array_equal(h[64: 64 + d], want.out)
    assert (h[:64] == 7.0).all() and (h[64 + d:] == 7.0).all()
    bits = torch.full(((d + 31) // 32,), -1, device=DEV, dtype=torch.int32)
    B.brace_vote_1bit(votes, d, 0, lam, out_bits=bits)           # bits only
    torch.cuda.synchronize()
    assert np.array_equal(bits.cpu().numpy().view(np.uint8)[: (d + 7) // 8], want.bits)


@pytest.mark.parametrize("n,d", [(3, 3), (7, 3), (5, 1024), (10, 10_000), (20, 100_003), (13, 4096),
                                 (6, 70_001), (37, 300_007), (100, 250_000)])
def test_one_bit_chunk_runs_tile_the_whole(n, d):
    g = special(n, d, seed=n + d)
    upd = to_device(g)
    for zs, lam in ((1, 1.0), (-1, -2.0)):
        votes = torch.empty(n, B.brace_1bit_row_words(d), device=DEV, dtype=torch.int32)
        B.brace_quantize_1bit(upd, zs, votes)
        want = O.brace_direct(g, lam, zs)
        out = torch.full((d,), 7.0, device=DEV, dtype=torch.float32)
        bits = torch.zeros((d + 31) // 32, device=DEV, dtype=torch.int32)
        for c in np.random.default_rng(n).permutation(n):       # chunk by chunk, scrambled
            B.brace_vote_1bit_chunks(votes, d, 0, int(c), int(c) + 1, lam, out=out, out_bits=bits)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), want.out), (n, d, zs)
        got_bits = bits.cpu().numpy().view(np.uint8)
        assert np.array_equal(got_bits[: (d + 7) // 8], want.bits)
        assert not got_bits[(d + 7) // 8:].any()
        guard = torch.full((d + 128,), 7.0, device=DEV, dtype=torch.float32)
        out2 = guard[64: 64 + d]
        a, b = n // 3, max(n // 3 + 1, (2 * n) // 3)            # one run in the middle, floats only
        B.brace_vote_1bit_chunks(votes, d, 0, a, b, lam, out=out2)
        torch.cuda.synchronize()
        lo, hi = O.chunk_range(n, d, a)[0], O.chunk_range(n, d, b - 1)[1]
        h = guard.cpu().numpy()
        assert np.array_equal(h[64 + lo: 64 + hi], want.out[lo:hi])
        assert (h[: 64 + lo] == 7.0).all() and (h[64 + hi:] == 7.0).all()


@pytest.mark.parametrize("idx,col_tile", [(2, 2_000_000), (3, 2_000_000), (4, 4_000_000)])
def test_one_bit_large_workloads_full(idx, col_tile):
    w = synth.WORKLOADS[idx]
    upd = synth.generate(w, DEV)
    zs = 1 if idx != 3 else -1
    # rows at the recommended pitch (whole 128-byte lines): the layout bench.py times
    vw, vp = B.brace_1bit_row_words(w.d), B.brace_1bit_row_pitch(w.d)
    assert vp % 32 == 0 and 0 <= vp - vw < 32
    votes = torch.full((w.n, vp), -1, device=DEV, dtype=torch.int32)[:, :vw]
    B.brace_quantize_1bit(upd, zs, votes)
    out = torch.empty(w.d, device=DEV, dtype=torch.float32)
    bits = torch.empty((w.d + 31) // 32, device=DEV, dtype=torch.int32)
    B.brace_vote_1bit(votes, w.d, w.f, 5.0, out=out, out_bits=bits)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    got_bits = bits.cpu().numpy().view(np.uint8)
    plane = votes.cpu().numpy().view(np.uint32)
    for k0 in range(0, w.d, col_tile):
        k1 = min(w.d, k0 + col_tile)
        host = upd[:, k0:k1].contiguous().cpu().numpy()
        want, _, _ = C.brace_direct(host, 5.0, zs, want_sums=False, want_bits=False)
        assert np.array_equal(got[k0:k1], want), (w.name, k0)
        assert np.array_equal(got_bits[k0 // 8: (k1 + 7) // 8], O.pack_bits(want)), (w.name, k0)
        # the votes themselves on the first and last coordinates of the tile
        s1 = min(k1, k0 + 262_144)
        ref = O.vote_plane(host[:, : s1 - k0], zs)
        nw = (s1 - k0) // 32
        assert np.array_equal(plane[:, k0 // 32: k0 // 32 + nw], ref[:, :nw]), (w.name, k0)
        s0 = max(k0, (k1 - 65_536) // 128 * 128)
        ref = O.vote_plane(host[:, s0 - k0:], zs)
        assert np.array_equal(plane[:, s0 // 32: s0 // 32 + ref.shape[1]], ref), (w.name, k0)
        print(f"{w.name}: one-bit vote over columns [{k0}, {k1}) matches", flush=True)
    del upd, votes
    torch.cuda.empty_cache()
