"""GPU parity for Phase III as its own call (brace_consensus_sums): Eq. (1) applied to partial
sign-sums, as a chunk owner applies it to what Share-Reduce delivered (Sec. 3), bit for bit
against the CPU oracle; and the phases chained on the GPU against the one-pass definition."""

import numpy as np
import pytest
import torch

from oracle import brace_oracle as O
from paper_2501_17392_amd import binding as B

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module", autouse=True)
def _gpu_and_library():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    B.lib()
    B.brace_reset_tuning()
    yield
    B.brace_reset_tuning()


def device_parts(parts, ld, offset):
    g, d = parts.shape
    store = torch.full((g * ld + offset + 16,), 77, device=DEV, dtype=torch.int16)
    view = store[offset: offset + g * ld].view(g, ld)[:, :d]
    view.copy_(torch.from_numpy(parts))
    return view


def run_consensus(parts_dev, d, lam, want_out=True, want_bits=True, out_off=0):
    whole = torch.full((d + 128 + out_off,), 7.0, device=DEV, dtype=torch.float32)
    out = whole[64 + out_off: 64 + out_off + d] if want_out else None
    bits = torch.full(((d + 31) // 32,), -1, device=DEV, dtype=torch.int32) if want_bits else None
    B.brace_consensus_sums(parts_dev, lam, out=out, out_bits=bits)
    torch.cuda.synchronize()
    h = whole.cpu().numpy()
    assert (h[: 64 + out_off] == 7.0).all() and (h[64 + out_off + d:] == 7.0).all()
    return (h[64 + out_off: 64 + out_off + d] if want_out else None,
            None if bits is None else np.unpackbits(bits.cpu().numpy().view(np.uint8), bitorder="little"))


@pytest.mark.parametrize("g,d,ld,offset,out_off", [
    (1, 1, None, 0, 0), (1, 300, None, 0, 0), (2, 7, None, 0, 0), (3, 8, None, 0, 0), (3, 9, None, 0, 0),
    (4, 31, None, 0, 0), (4, 32, None, 0, 0), (5, 33, None, 0, 0), (8, 1000, None, 0, 0),
    (8, 4099, 4104, 0, 0),      # padded pitch, 16-byte rows: wide path with a ragged tail
    (8, 4099, 4100, 0, 0),      # rows not 16-byte aligned: one coordinate per thread
    (5, 12_345, None, 1, 0), (5, 12_344, None, 0, 1), (9, 70_001, 70_008, 0, 0), (16, 262_144, None, 0, 0)])
def test_consensus_of_partial_sums_matches_oracle(g, d, ld, offset, out_off):
    rng = np.random.default_rng(g * 131 + d)
    parts = rng.integers(-40, 41, size=(g, d)).astype(np.int16)
    parts[:, : min(d, 5)] = np.array([32767, -32767, 0, 1, -1], dtype=np.int16)[: min(d, 5)]   # extremes
    dev = device_parts(parts, d if ld is None else ld, offset)
    total = parts.astype(np.int64).sum(axis=0)
    for lam in (-1e12, -3.0, -0.5, 0.0, 0.5, 5.0, float(g * 20), float(g) * 32767.0, 1e12):
        want = O.consensus(total, lam)
        out, unpacked = run_consensus(dev, d, lam, out_off=out_off)
        assert np.array_equal(out, want), (g, d, lam)
        assert np.array_equal(unpacked[:d], (want > 0).astype(np.uint8)), (g, d, lam)
        assert not unpacked[d:].any(), "padding bits must be zero"
    want = O.consensus(total, 1.0)
    out, _ = run_consensus(dev, d, 1.0, want_bits=False, out_off=out_off)
    assert np.array_equal(out, want)
    _, unpacked = run_consensus(dev, d, 1.0, want_out=False)
    assert np.array_equal(unpacked[:d], (want > 0).astype(np.uint8)) and not unpacked[d:].any()


@pytest.mark.parametrize("n,groups,d", [(12, 3, 10_000), (20, 4, 100_003), (9, 9, 4097), (7, 1, 5000)])
def test_phases_chained_on_the_gpu_equal_the_one_pass_vote(n, groups, d):
    """Phase I+II per group of clients (sign-sums of brace_aggregate), Phase III on the partial
    sums, Phase IV from the packed bits: the same vector as the definition on all n clients."""
    rng = np.random.default_rng(n * 7 + d)
    gmat = rng.standard_normal((n, d)).astype(np.float32)
    gmat[rng.random((n, d)) < 0.1] = 0.0
    gmat[rng.random((n, d)) < 0.02] = np.nan
    upd = torch.from_numpy(gmat).to(DEV)
    cuts = [round(j * n / groups) for j in range(groups + 1)]
    for zs in (0, 1, -1):
        parts = torch.empty((groups, d), device=DEV, dtype=torch.int16)
        for j in range(groups):
            B.brace_aggregate(upd[cuts[j]: cuts[j + 1]], 0, 0.0, zs, sums=parts[j])
        torch.cuda.synchronize()
        # the partial sums themselves are what the oracle's Phase I + II give for each group
        for j in range(groups):
            ref = O.sign_quantize(gmat[cuts[j]: cuts[j + 1]], zs).sum(axis=0)
            assert np.array_equal(parts[j].cpu().numpy().astype(np.int64), ref)
        for lam in (-1.0, 0.0, 2.0, 5.0):
            want = O.brace_direct(gmat, lam, zs)
            bits = torch.empty((d + 31) // 32, device=DEV, dtype=torch.int32)
            B.brace_consensus_sums(parts, lam, out_bits=bits)
            out = torch.empty(d, device=DEV, dtype=torch.float32)
            B.brace_expand_bits(bits, d, out)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy(), want.out), (n, groups, d, zs, lam)
            assert np.array_equal(bits.cpu().numpy().view(np.uint8)[: (d + 7) // 8], want.bits)


@pytest.mark.parametrize("n,d,ld,offset,soff", [
    (1, 1, None, 0, 0), (3, 1024, None, 0, 0), (5, 8192 * 3 + 5, None, 0, 0), (12, 100_003, None, 0, 0),
    (12, 100_003, 100_004, 0, 0), (12, 100_002, None, 0, 0), (7, 70_001, None, 1, 0),
    (9, 50_000, None, 0, 1), (9, 50_000, None, 0, 2), (9, 50_000, None, 0, 4), (40, 300_007, None, 0, 0)])
@pytest.mark.parametrize("stage", [0, 1, 2], ids=["auto", "per-wave-stores", "bursts"])
def test_sign_sums_alone_match_the_oracle(n, d, ld, offset, soff, stage):
    """Phase I + II delivered as data (what a device contributes to Share-Reduce): the int16
    sign-sums as the only output, with per-wave stores and with LDS-staged bursts."""
    rng = np.random.default_rng(n * 17 + d + soff)
    g = rng.standard_normal((n, d)).astype(np.float32)
    g[rng.random((n, d)) < 0.1] = 0.0
    g[rng.random((n, d)) < 0.03] = -0.0
    g[rng.random((n, d)) < 0.02] = np.nan
    ld = d if ld is None else ld
    store = torch.full((n * ld + offset + 8,), float("nan"), device=DEV, dtype=torch.float32)
    upd = store[offset: offset + n * ld].view(n, ld)[:, :d]
    upd.copy_(torch.from_numpy(g))
    for zs in (0, 1, -1):
        whole = torch.full((d + 128 + soff,), 12345, device=DEV, dtype=torch.int16)
        sums = whole[64 + soff: 64 + soff + d]
        try:
            B.brace_set_tuning(stage_writes=stage)
            B.brace_aggregate(upd, 0, 0.0, zs, sums=sums)
        finally:
            B.brace_reset_tuning()
        torch.cuda.synchronize()
        h = whole.cpu().numpy()
        want = O.sign_quantize(g, zs).sum(axis=0)
        assert np.array_equal(h[64 + soff: 64 + soff + d].astype(np.int64), want), (n, d, zs, stage)
        assert (h[: 64 + soff] == 12345).all() and (h[64 + soff + d:] == 12345).all()
