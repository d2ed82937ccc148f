"""GPU parity: the HIP path through the C ABI against the CPU oracle, bit for bit.

Every output of the path is a selection result or an integer (+-1.0f, packed bits,
int16 sign-sums), so the bar is exact equality on the same input bytes.  Inputs are
generated once (on the device for the large workloads) and the oracle reads a copy of
those bytes; nothing is regenerated per side.
"""

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
    B.lib()                      # raises if libbrace.so was not built: no fallback
    B.brace_reset_tuning()
    yield
    B.brace_reset_tuning()


def lambda_sweep(n, f):
    return sorted({-n - 1.0, -1.0, 0.0, 0.5, 1.0, 2.0, 5.0, float(f), float(n - f), float(n)})


def gpu_aggregate(upd, f, lam, zs=0, want_bits=True, want_sums=True, chunk=None, bufs=None):
    """Run the C ABI on a device matrix; returns (out, bits, sums) as numpy (None if not asked)."""
    n, d = upd.shape
    if bufs is None:
        out = torch.full((d,), 7.0, device=DEV, dtype=torch.float32)
        bits = torch.full(((d + 31) // 32,), -1, device=DEV, dtype=torch.int32) if want_bits else None
        sums = torch.full((d,), 12345, device=DEV, dtype=torch.int16) if want_sums else None
    else:
        out, bits, sums = bufs
    if chunk is None:
        B.brace_aggregate(upd, f, lam, zs, out=out, out_bits=bits, sums=sums)
    else:
        B.brace_aggregate_chunk(upd, f, chunk, lam, zs, out=out, out_bits=bits, sums=sums)
    torch.cuda.synchronize()
    return (out.cpu().numpy(),
            None if bits is None else bits.cpu().numpy().view(np.uint8),
            None if sums is None else sums.cpu().numpy())


def check_against_oracle(upd, f, lam, zs=0):
    n, d = upd.shape
    host = upd.cpu().numpy()
    want = O.brace_direct(host, lam, zs)
    out, bits, sums = gpu_aggregate(upd, f, lam, zs)
    assert np.array_equal(out, want.out), f"out differs (n={n}, d={d}, lam={lam}, zs={zs})"
    assert np.array_equal(sums.astype(np.int64), want.sums)
    nb = (d + 7) // 8
    assert np.array_equal(bits[:nb], want.bits)
    assert not bits[nb:].any(), "padding bytes of the last 32-bit word must be zero"


def special_matrix(n, d, seed, ld=None, offset=0):
    """Random matrix with zeros, negative zeros, NaN, infinities and denormals mixed in,
    placed in a pitched allocation that starts `offset` elements past an aligned address."""
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
    ld = d if ld is None else ld
    store = torch.full((n * max(ld, 1) + offset + 8,), float("nan"), device=DEV, dtype=torch.float32)
    view = store[offset: offset + n * max(ld, 1)].view(n, max(ld, 1))[:, :d]
    view.copy_(torch.from_numpy(g))
    return view


# --------------------------------------------------------------------------
# Small shapes: several tiles, ragged tails, every alignment class, special values
# --------------------------------------------------------------------------

SHAPES = [
    # n, d, ld, offset
    (1, 1, None, 0), (1, 300, None, 0), (2, 5, None, 0), (3, 63, None, 0), (3, 64, None, 0),
    (3, 65, None, 0), (5, 255, None, 0), (5, 256, None, 0), (5, 257, None, 0),
    (7, 1000, None, 0), (10, 4099, None, 0), (33, 70_001, None, 0), (100, 20_000, None, 0),
    (8, 5000, 5004, 0),        # padded pitch, 16-byte rows
    (8, 5000, 5002, 0),        # 8-byte rows
    (8, 5000, 5001, 0),        # 4-byte rows
    (9, 12_345, None, 1), (9, 12_345, None, 2), (9, 12_344, None, 3),   # base pointer off 16 B
    (20, 50_003, None, 0), (6, 2048 * 3 + 17, None, 0),
]


@pytest.mark.parametrize("n,d,ld,offset", SHAPES)
def test_small_shapes_bit_exact(n, d, ld, offset):
    upd = special_matrix(n, d, seed=n * 1000 + d, ld=ld, offset=offset)
    for lam in (-1.0, 0.0, 2.0, 5.0):
        for zs in (0, 1, -1):
            check_against_oracle(upd, 0, lam, zs)


@pytest.mark.parametrize("n,d", [(1000, 700), (4097, 300), (32767, 130)])
def test_many_clients(n, d):
    # n up to the ABI limit (sign-sums are int16): counters, row split and int16 sums hold.
    upd = special_matrix(n, d, seed=n)
    f = n // 5
    for lam in (0.0, 5.0, float(f), float(n - 1), -float(n)):
        check_against_oracle(upd, f, lam)
    ones = torch.ones(n, d, device=DEV)
    out, bits, sums = gpu_aggregate(ones, 0, n - 1.0)
    assert (sums == n).all() and (out == 1.0).all()          # S = n exactly, > n - 1
    out, bits, sums = gpu_aggregate(-ones, 0, -float(n) - 0.5)
    assert (sums == -n).all() and (out == 1.0).all()         # S = -n > -n - 0.5


def test_lambda_sweep_bit_exact():
    n, f, d = 25, 5, 9001
    upd = special_matrix(n, d, seed=77)
    for lam in lambda_sweep(n, f) + [4.999, -0.5, 1e30, -1e30]:
        check_against_oracle(upd, f, lam)


def test_optional_outputs_are_optional():
    n, d = 12, 3001
    upd = special_matrix(n, d, seed=5)
    want = O.brace_direct(upd.cpu().numpy(), 2.0)
    out, bits, sums = gpu_aggregate(upd, 0, 2.0, want_bits=False, want_sums=False)
    assert np.array_equal(out, want.out) and bits is None and sums is None
    bits_t = torch.zeros((d + 31) // 32, device=DEV, dtype=torch.int32)
    B.brace_aggregate(upd, 0, 2.0, out=None, out_bits=bits_t)       # packed-only output
    torch.cuda.synchronize()
    assert np.array_equal(bits_t.cpu().numpy().view(np.uint8)[: (d + 7) // 8], want.bits)
    sums_t = torch.zeros(d, device=DEV, dtype=torch.int16)
    B.brace_aggregate(upd, 0, 2.0, out=None, sums=sums_t)
    torch.cuda.synchronize()
    assert np.array_equal(sums_t.cpu().numpy().astype(np.int64), want.sums)


def test_empty_input_is_a_no_op():
    upd = torch.empty(4, 0, device=DEV, dtype=torch.float32)
    out = torch.empty(0, device=DEV, dtype=torch.float32)
    B.brace_aggregate(upd, 1, 5.0, out=out)
    torch.cuda.synchronize()


def test_padding_never_leaks_into_the_result():
    # NaN padding between rows and a guard band around `out` must stay untouched / unread.
    n, d, ld = 6, 1500, 1536
    upd = special_matrix(n, d, seed=9, ld=ld)
    guard = torch.full((d + 64,), 3.0, device=DEV, dtype=torch.float32)
    out = guard[32: 32 + d]
    B.brace_aggregate(upd, 0, 0.0, out=out)
    torch.cuda.synchronize()
    g = guard.cpu().numpy()
    assert (g[:32] == 3.0).all() and (g[32 + d:] == 3.0).all()
    assert np.array_equal(g[32: 32 + d], O.brace_direct(upd.cpu().numpy(), 0.0).out)


@pytest.mark.parametrize("n,d", [(5, 1024), (7, 8192 * 3 + 5), (12, 100_003), (100, 40_000)])
def test_staged_float_output_forced(n, d):
    # float-only output through the LDS-staged kernel (no bits, no sums, writes not split)
    upd = special_matrix(n, d, seed=n + d)
    host = upd.cpu().numpy()
    try:
        B.brace_set_tuning(split_writes=1, stage_writes=2)
        for lam, rule in ((2.0, 0), (0.0, 1)):
            guard = torch.full((d + 64,), 3.0, device=DEV, dtype=torch.float32)
            out = guard[32: 32 + d]
            B.brace_aggregate(upd, 0, lam, out=out, rule=rule)
            torch.cuda.synchronize()
            g = guard.cpu().numpy()
            want = O.signsgd_majority(host) if rule else O.brace_direct(host, lam).out
            assert np.array_equal(g[32: 32 + d], want)
            assert (g[:32] == 3.0).all() and (g[32 + d:] == 3.0).all()
    finally:
        B.brace_reset_tuning()


def test_majority_rule_three_valued():
    # signSGD's plain majority over the same four phases: ties stay at 0.
    for n, d in ((4, 5000), (7, 3001), (10, 70_001)):
        upd = special_matrix(n, d, seed=n)
        host = upd.cpu().numpy()
        for zs in (0, 1, -1):
            want = O.signsgd_majority(host, zs)
            out = torch.full((d,), 7.0, device=DEV, dtype=torch.float32)
            sums = torch.zeros(d, device=DEV, dtype=torch.int16)
            B.brace_aggregate(upd, 0, 123.0, zs, out=out, sums=sums, rule=1)   # lambda is ignored
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy(), want), (n, d, zs)
            assert np.array_equal(sums.cpu().numpy().astype(np.int64), O.brace_direct(host, 0.0, zs).sums)
            parts = torch.full((d,), 7.0, device=DEV, dtype=torch.float32)
            for c in range(n):
                B.brace_aggregate_chunk(upd, 0, c, 0.0, zs, out=parts, rule=1)
            torch.cuda.synchronize()
            assert np.array_equal(parts.cpu().numpy(), want)
        if n == 4:
            assert (want == 0).any()
        w0 = torch.randn(d, device=DEV)
        w = w0.clone()
        B.brace_aggregate_update(upd, 0, w, 0.5, 0.0, rule=1)
        torch.cuda.synchronize()
        want_w = O.model_update(w0.cpu().numpy(), O.signsgd_majority(host), 0.5)
        assert np.allclose(w.cpu().numpy(), want_w, rtol=1e-5, atol=1e-6)
    with pytest.raises(B.BraceError):
        B.brace_aggregate(upd, 0, 0.0, out=out, out_bits=torch.zeros(4000, device=DEV, dtype=torch.int32),
                          rule=1)


# --------------------------------------------------------------------------
# Per-chunk entry point: union of the chunks == whole, byte for byte
# --------------------------------------------------------------------------

@pytest.mark.parametrize("n,d", [(3, 3), (7, 3), (10, 10_000), (20, 100_003), (13, 4096),
                                 (100, 25_000), (5, 1)])
def test_chunks_tile_the_whole(n, d):
    upd = special_matrix(n, d, seed=n + d)
    lam = 1.0
    whole = gpu_aggregate(upd, 0, lam)
    out = torch.full((d,), 7.0, device=DEV, dtype=torch.float32)
    bits = torch.full(((d + 31) // 32,), -1, device=DEV, dtype=torch.int32)
    sums = torch.full((d,), 12345, device=DEV, dtype=torch.int16)
    # odd chunks on a second stream: neighbouring chunks may share a 32-bit word of bits
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    for c in range(n):
        if c % 2:
            with torch.cuda.stream(side):
                B.brace_aggregate_chunk(upd, 0, c, lam, out=out, out_bits=bits, sums=sums)
        else:
            B.brace_aggregate_chunk(upd, 0, c, lam, out=out, out_bits=bits, sums=sums)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), whole[0])
    assert np.array_equal(bits.cpu().numpy().view(np.uint8), whole[1])
    assert np.array_equal(sums.cpu().numpy(), whole[2])
    want = O.brace_direct(upd.cpu().numpy(), lam)
    assert np.array_equal(whole[0], want.out)


def test_runs_of_chunks_tile_the_whole():
    # eight "devices" each taking a run of consecutive chunks
    n, d = 100, 250_007
    upd = special_matrix(n, d, seed=12)
    want = O.brace_direct(upd.cpu().numpy(), 2.0)
    out = torch.full((d,), 7.0, device=DEV, dtype=torch.float32)
    bits = torch.full(((d + 31) // 32,), -1, device=DEV, dtype=torch.int32)
    sums = torch.full((d,), 12345, device=DEV, dtype=torch.int16)
    cuts = [0, 13, 25, 38, 50, 63, 75, 88, 100]
    for a, b in zip(cuts[:-1], cuts[1:]):
        B.brace_aggregate_chunks(upd, 20, a, b, 2.0, out=out, out_bits=bits, sums=sums)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), want.out)
    assert np.array_equal(sums.cpu().numpy().astype(np.int64), want.sums)
    assert np.array_equal(bits.cpu().numpy().view(np.uint8)[: (d + 7) // 8], want.bits)
    lo, _ = B.brace_chunk_range(n, d, 13)
    _, hi = B.brace_chunk_range(n, d, 24)
    part = torch.full((d,), 7.0, device=DEV, dtype=torch.float32)
    B.brace_aggregate_chunks(upd, 20, 13, 25, 2.0, out=part)
    torch.cuda.synchronize()
    p = part.cpu().numpy()
    assert np.array_equal(p[lo:hi], want.out[lo:hi]) and (p[:lo] == 7).all() and (p[hi:] == 7).all()


def test_single_chunk_touches_only_its_range():
    n, d, c = 10, 10_007, 4
    upd = special_matrix(n, d, seed=3)
    out, bits, sums = gpu_aggregate(upd, 0, 0.0, chunk=c)
    lo, hi = B.brace_chunk_range(n, d, c)
    assert (lo, hi) == O.chunk_range(n, d, c)
    _, _, want_out, want_sums = O.brace_chunk(upd.cpu().numpy(), c, 0.0)
    assert np.array_equal(out[lo:hi], want_out)
    assert np.array_equal(sums[lo:hi].astype(np.int64), want_sums)
    assert (out[:lo] == 7.0).all() and (out[hi:] == 7.0).all()
    assert (sums[:lo] == 12345).all() and (sums[hi:] == 12345).all()
    got_bits = np.unpackbits(bits, bitorder="little")[:d]
    assert np.array_equal(got_bits[lo:hi], (want_out > 0).astype(np.uint8))
    assert got_bits[:lo].all() and got_bits[hi:].all()      # untouched bits keep their 1s


@pytest.mark.parametrize("n,d,offset", [(5, 1024, 0), (5, 1023, 0), (7, 5000, 0), (9, 40_000, 4),
                                        (9, 40_001, 8), (3, 2048 + 1, 0), (12, 100_003, 0)])
def test_split_write_path_bit_exact(n, d, offset):
    # Force the two-kernel path (bits first, floats expanded afterwards) on small inputs,
    # with and without a separate bit array (without it the bit-words are parked in `out`).
    upd = special_matrix(n, d, seed=n * 31 + d)
    want = O.brace_direct(upd.cpu().numpy(), 1.0)
    try:
        B.brace_set_tuning(split_writes=2)
        guard = torch.full((d + 64 + offset,), 3.0, device=DEV, dtype=torch.float32)
        out = guard[32 + offset: 32 + offset + d]
        for with_bits in (False, True):
            guard.fill_(3.0)
            bits = torch.full(((d + 31) // 32,), -1, device=DEV, dtype=torch.int32) if with_bits else None
            B.brace_aggregate(upd, 0, 1.0, out=out, out_bits=bits)
            torch.cuda.synchronize()
            g = guard.cpu().numpy()
            assert np.array_equal(g[32 + offset: 32 + offset + d], want.out), with_bits
            assert (g[: 32 + offset] == 3.0).all() and (g[32 + offset + d:] == 3.0).all()
            if with_bits:
                assert np.array_equal(bits.cpu().numpy().view(np.uint8)[: (d + 7) // 8], want.bits)
        # chunk by chunk through the same forced path
        chunked = torch.full((d,), 7.0, device=DEV, dtype=torch.float32)
        for c in range(n):
            B.brace_aggregate_chunk(upd, 0, c, 1.0, out=chunked)
        torch.cuda.synchronize()
        assert np.array_equal(chunked.cpu().numpy(), want.out)
    finally:
        B.brace_reset_tuning()


# --------------------------------------------------------------------------
# Every launch tuning computes the same thing
# --------------------------------------------------------------------------

def test_all_tunings_agree_with_the_oracle():
    n, d = 37, 300_007
    try:
        for ld, off in ((d + 1, 0), (d + 3, 0), (d, 0), (d + 1, 1)):   # 16 B, 8 B, 4 B rows; odd base
            view = special_matrix(n, d, seed=ld + off, ld=ld, offset=off)
            want = O.brace_direct(view.cpu().numpy(), 2.0)
            for vec in (0, 1, 2, 4):
                for cols in (1, 2, 4, 8):
                    for unroll in (2, 4, 8):
                        for nt, pipe, split, rs in ((0, 0, 1, 1), (1, 0, 2, 2), (1, 1, 1, 2),
                                                    (0, 1, 2, 1), (1, 1, 0, 0)):
                            B.brace_set_tuning(vec, cols, unroll, nt, pipe, split, rs)
                            out, bits, sums = gpu_aggregate(view, 0, 2.0)
                            tag = (ld, off, vec, cols, unroll, nt, pipe, split, rs)
                            assert np.array_equal(out, want.out), tag
                            assert np.array_equal(sums.astype(np.int64), want.sums), tag
                            assert np.array_equal(bits[: (d + 7) // 8], want.bits), tag
                            out, _, _ = gpu_aggregate(view, 0, 2.0, want_bits=False,
                                                      want_sums=False)
                            assert np.array_equal(out, want.out), tag
    finally:
        B.brace_reset_tuning()


# --------------------------------------------------------------------------
# The five workloads at full size
# --------------------------------------------------------------------------

def test_cfg0_full_against_definition_and_ring_simulation():
    w = synth.WORKLOADS[0]
    upd = synth.generate(w, DEV)
    host = upd.cpu().numpy()
    for lam in lambda_sweep(w.n, w.f):
        check_against_oracle(upd, w.f, lam)
    ring = O.ring_all_reduce(host, mode="brace", lam=5.0)
    out, _, _ = gpu_aggregate(upd, w.f, 5.0)
    for b in ring.buffers:
        assert np.array_equal(out, b)
    # rows in another order: same result (permutation invariance)
    perm = torch.randperm(w.n, generator=torch.Generator().manual_seed(0)).to(DEV)
    out_p, _, _ = gpu_aggregate(upd[perm].contiguous(), w.f, 5.0)
    assert np.array_equal(out_p, out)


def test_cfg1_full_unequal_chunks():
    w = synth.WORKLOADS[1]
    upd = synth.generate(w, DEV)
    host = upd.cpu().numpy()
    for lam in (0.0, 5.0, float(w.f), float(w.n - w.f)):
        want = O.brace_direct(host, lam)
        out, bits, sums = gpu_aggregate(upd, w.f, lam)
        assert np.array_equal(out, want.out)
        assert np.array_equal(sums.astype(np.int64), want.sums)
        assert np.array_equal(bits[: (w.d + 7) // 8], want.bits)
    ring = O.ring_all_reduce(host, mode="brace", lam=5.0)
    out5, _, _ = gpu_aggregate(upd, w.f, 5.0)
    assert np.array_equal(out5, ring.buffers[0]) and np.array_equal(out5, ring.buffers[-1])
    # chunk by chunk (3 chunks of 50,001 then 17 of 50,000)
    out = torch.full((w.d,), 7.0, device=DEV, dtype=torch.float32)
    for c in range(w.n):
        B.brace_aggregate_chunk(upd, w.f, c, 5.0, out=out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), out5)


def _full_size_check(w, lams, col_tile=2_000_000):
    """Whole workload on the GPU in the default (benchmark) launch configuration; the C oracle
    walks the same bytes in column tiles copied back from the device."""
    upd = synth.generate(w, DEV)
    results = {}
    for lam in lams:
        out = torch.empty(w.d, device=DEV, dtype=torch.float32)
        sums = torch.empty(w.d, device=DEV, dtype=torch.int16)
        bits = torch.empty((w.d + 31) // 32, device=DEV, dtype=torch.int32)
        B.brace_aggregate(upd, w.f, lam, out=out, out_bits=bits, sums=sums)
        out_only = torch.empty(w.d, device=DEV, dtype=torch.float32)
        B.brace_aggregate(upd, w.f, lam, out=out_only)           # the launch bench.py times
        torch.cuda.synchronize()
        assert torch.equal(out, out_only)
        results[lam] = (out.cpu().numpy(), sums.cpu().numpy(), bits.cpu().numpy().view(np.uint8))
    mixed = 0
    for k0 in range(0, w.d, col_tile):
        k1 = min(w.d, k0 + col_tile)
        host = upd[:, k0:k1].contiguous().cpu().numpy()
        for lam in lams:
            want_out, want_sums, _ = C.brace_direct(host, lam, 0, want_bits=False)
            out, sums, bits = results[lam]
            assert np.array_equal(out[k0:k1], want_out), (w.name, lam, k0)
            assert np.array_equal(sums[k0:k1], want_sums.astype(np.int16)), (w.name, lam, k0)
            assert k0 % 8 == 0
            assert np.array_equal(bits[k0 // 8: (k1 + 7) // 8], O.pack_bits(want_out)), (w.name, lam, k0)
            mixed += int((want_out > 0).sum())
        print(f"{w.name}: columns [{k0}, {k1}) match", flush=True)
    del upd
    torch.cuda.empty_cache()
    return mixed


def test_cfg2_full_resnet18_sized():
    w = synth.WORKLOADS[2]
    assert _full_size_check(w, (5.0, 0.0)) > 0


def test_cfg3_full_headline():
    w = synth.WORKLOADS[3]
    assert _full_size_check(w, (5.0, float(w.f))) > 0


def test_cfg4_full_sparse_mix():
    w = synth.WORKLOADS[4]
    assert _full_size_check(w, (5.0,), col_tile=4_000_000) > 0


# --------------------------------------------------------------------------
# Host-side buffer checks: a wrong shape is an error code, not a GPU fault
# --------------------------------------------------------------------------

def test_wrong_buffers_are_rejected_on_the_host():
    small = torch.zeros(1000, device=DEV)
    out = torch.zeros(1000, device=DEV)
    import ctypes
    # one client, but a dimension far beyond what the buffers hold
    with pytest.raises(B.BraceError) as ei:
        bits = torch.zeros(200_000_000 // 32, device=DEV, dtype=torch.int32)
        p = B.make_params(5.0, 0, 0, bits.data_ptr(), None)
        B._check(B.lib().brace_aggregate(small.data_ptr(), 1, 200_000_000, 0, ctypes.byref(p),
                                         None, None))
    assert ei.value.code == B.BRACE_EINVAL and "allocation" in ei.value.text
    big = torch.zeros(4, 100_000, device=DEV)
    with pytest.raises(B.BraceError) as ei:                    # out too short for d
        p = B.make_params(5.0, 0, 100_000, None, None)
        rc = B.lib().brace_aggregate(big.data_ptr(), 4, 100_000_000, 0, ctypes.byref(p),
                                     out.data_ptr(), None)
        B._check(rc)
    assert ei.value.code == B.BRACE_EINVAL
    pinned = torch.zeros(1000, pin_memory=True)
    with pytest.raises(B.BraceError) as ei:                    # host memory is not accepted
        p = B.make_params(5.0, 0, 0, None, None)
        B._check(B.lib().brace_aggregate(big.data_ptr(), 4, 1000, 0, ctypes.byref(p),
                                         pinned.data_ptr(), None))
    assert ei.value.code == B.BRACE_EINVAL
    with pytest.raises(B.BraceError):
        B.brace_expand_bits(torch.zeros(4, device=DEV, dtype=torch.int32), 200_000_000, out)
    # nothing above launched anything or left an error behind: a good call still works
    good = torch.empty(100_000, device=DEV)
    B.brace_aggregate(big, 0, 0.0, out=good)
    torch.cuda.synchronize()
    assert (good == -1.0).all()
    # switched off, the same good call works too
    B.brace_set_pointer_checks(False)
    try:
        B.brace_aggregate(big, 0, -1.0, out=good)
        torch.cuda.synchronize()
        assert (good == 1.0).all()
    finally:
        B.brace_set_pointer_checks(True)


def test_calls_from_several_host_threads():
    """Four host threads, each with its own stream, inputs and outputs, call the entry points
    at the same time (ctypes releases the interpreter lock during a call); every result must
    match the oracle and an error on one thread must not leak its text to another."""
    import threading
    n, d = 9, 120_003
    inputs = [special_matrix(n, d, seed=500 + t) for t in range(4)]
    wants = [O.brace_direct(v.cpu().numpy(), 1.0) for v in inputs]
    sums_ref = [O.rar_sum_direct(np.nan_to_num(v.cpu().numpy(), nan=0.0, posinf=0.0, neginf=0.0))
                for v in inputs]
    clean = [torch.nan_to_num(v, nan=0.0, posinf=0.0, neginf=0.0).contiguous() for v in inputs]
    failures = []

    def worker(t):
        try:
            stream = torch.cuda.Stream()
            out = torch.empty(d, device=DEV, dtype=torch.float32)
            total = torch.empty(d, device=DEV, dtype=torch.float32)
            bits = torch.empty((d + 31) // 32, device=DEV, dtype=torch.int32)
            for it in range(25):
                B.brace_aggregate(inputs[t], 0, 1.0, out=out, out_bits=bits, stream=stream)
                B.brace_rar_aggregate(clean[t], total, stream=stream)
                if it % 5 == t % 5:
                    with pytest.raises(B.BraceError) as err:     # an error of this thread's own
                        B.brace_aggregate_chunk(inputs[t], 0, n + t, 1.0, out=out, stream=stream)
                    assert f"chunk {n + t} " in str(err.value)
            stream.synchronize()
            assert np.array_equal(out.cpu().numpy(), wants[t].out)
            assert np.array_equal(bits.cpu().numpy().view(np.uint8)[: (d + 7) // 8], wants[t].bits)
            got = total.cpu().numpy().astype(np.float64)
            assert np.all(np.abs(got - sums_ref[t]) <= 1e-6 + 1e-5 * np.abs(sums_ref[t]))
        except BaseException as e:                               # reported by the main thread
            failures.append((t, repr(e)))

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(4)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    torch.cuda.synchronize()
    assert not failures, failures


def test_binding_refuses_tensors_the_abi_would_misread():
    # The C side sees only addresses: element type, device and contiguity are the binding's to check.
    upd = torch.randn(4, 1000, device=DEV)
    out = torch.empty(1000, device=DEV)
    with pytest.raises(ValueError):
        B.brace_aggregate(upd, 0, 0.0, out=torch.empty(1000, device=DEV, dtype=torch.float64))
    with pytest.raises(ValueError):
        B.brace_aggregate(upd, 0, 0.0, out=torch.empty(1000))                    # host tensor
    with pytest.raises(ValueError):
        B.brace_aggregate(upd, 0, 0.0, out=torch.empty(2000, device=DEV)[::2])  # strided
    with pytest.raises(ValueError):
        B.brace_aggregate(upd, 0, 0.0, out=out, sums=torch.empty(1000, device=DEV, dtype=torch.int64))
    with pytest.raises(ValueError):
        B.brace_aggregate(upd.double(), 0, 0.0, out=out)
    with pytest.raises(ValueError):
        B.brace_aggregate(upd.t(), 0, 0.0, out=out)                              # column-major view
    with pytest.raises(ValueError):
        B.brace_vote_packed(torch.zeros(4, 64, device=DEV, dtype=torch.int64), 1000, 0, out=out)
    with pytest.raises(ValueError):
        B.brace_consensus_sums(torch.zeros(4, 1000, device=DEV, dtype=torch.int32), out=out)
    with pytest.raises(ValueError):
        B.brace_rar_aggregate(upd, torch.empty(1000, device=DEV, dtype=torch.float16))
    B.brace_aggregate(upd, 0, 0.0, out=out)                                      # a good call still works
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), O.brace_direct(upd.cpu().numpy(), 0.0).out)


def test_overlapping_buffers_of_one_call_are_rejected():
    # Every pair of buffers of a call must be disjoint (the split write path parks bit-words in
    # `out`, so an overlap would corrupt silently); the call answers EINVAL and launches nothing.
    n, d = 6, 40_000
    upd = torch.randn(n, d, device=DEV)
    out = torch.full((d,), 7.0, device=DEV)
    as_bits = out[:2048].view(torch.int32)                       # bit array inside out
    for kw in (dict(out=out, out_bits=as_bits),
               dict(out=out, sums=out[1000:1000 + d // 2].view(torch.int16)),
               dict(out=None, out_bits=as_bits, sums=out[:d // 2].view(torch.int16)),
               dict(out=None, out_bits=upd[2, :2048].view(torch.int32)),
               dict(out=None, sums=upd[n - 1, d // 2:].view(torch.int16))):
        with pytest.raises(B.BraceError) as ei:
            B.brace_aggregate(upd, 0, 0.0, **kw)
        assert ei.value.code == B.BRACE_EINVAL and "overlaps" in ei.value.text, kw
    w = torch.zeros(d, device=DEV)
    with pytest.raises(B.BraceError) as ei:
        B.brace_aggregate_update(upd, 0, w, 0.1, out_bits=w[:2048].view(torch.int32))
    assert "overlaps" in ei.value.text
    torch.cuda.synchronize()
    assert (out == 7.0).all() and (w == 0.0).all()              # nothing was written
