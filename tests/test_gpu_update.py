"""GPU parity for the vote fused with the model update, and for the receive side of Share-Only
(expand / apply the packed bits), against the CPU oracle.

The update is one fp32 operation per coordinate (w -+ eta), so against the oracle's fp64
`w - eta * result` it must sit within the floating-point bar |gpu - oracle| <= 1e-6 + 1e-5 |oracle|,
and in fact within one fp32 rounding of it.
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
RTOL, ATOL = 1e-5, 1e-6


@pytest.fixture(scope="module", autouse=True)
def _gpu_and_library():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    B.lib()
    B.brace_reset_tuning()
    yield
    B.brace_reset_tuning()


def check_update(got32, w_host32, agg, eta):
    want = O.model_update(w_host32, agg, np.float32(eta))
    got = got32.astype(np.float64)
    assert np.all(np.abs(got - want) <= ATOL + RTOL * np.abs(want))
    assert np.all(np.abs(got - want) <= np.spacing(np.abs(want).astype(np.float32)).astype(np.float64))


def matrix(n, d, seed, offset=0):
    rng = np.random.default_rng(seed)
    g = rng.standard_normal((n, d)).astype(np.float32)
    g[rng.random((n, d)) < 0.1] = 0.0
    g[rng.random((n, d)) < 0.02] = np.nan
    store = torch.empty(n * d + offset + 8, device=DEV, dtype=torch.float32)
    view = store[offset: offset + n * d].view(n, d)
    view.copy_(torch.from_numpy(g))
    return view


@pytest.mark.parametrize("n,d,offset,woff", [(1, 1, 0, 0), (3, 65, 0, 0), (7, 1000, 0, 0),
                                             (10, 4099, 0, 0), (33, 70_001, 0, 0), (9, 12_345, 1, 0),
                                             (9, 12_344, 0, 3), (20, 50_003, 0, 0), (12, 8192, 0, 4)])
def test_fused_update_small_shapes(n, d, offset, woff):
    upd = matrix(n, d, seed=n * 13 + d, offset=offset)
    host = upd.cpu().numpy()
    rng = np.random.default_rng(d)
    w0 = rng.standard_normal(d).astype(np.float32)
    for lam, eta, split, stage in ((2.0, 0.01, 0, 0), (0.0, 0.5, 2, 1), (-1.0, 1e-3, 2, 2),
                                   (1.0, 0.25, 1, 2)):
        agg = O.brace_direct(host, lam).out
        try:
            B.brace_set_tuning(split_writes=split, stage_writes=stage)
            for with_bits in (False, True):
                guard = torch.full((d + 16 + woff,), 5.0, device=DEV, dtype=torch.float32)
                w = guard[8 + woff: 8 + woff + d]
                w.copy_(torch.from_numpy(w0))
                bits = torch.full(((d + 31) // 32,), -1, device=DEV, dtype=torch.int32) if with_bits else None
                B.brace_aggregate_update(upd, 0, w, eta, lam, out_bits=bits)
                torch.cuda.synchronize()
                g = guard.cpu().numpy()
                check_update(g[8 + woff: 8 + woff + d], w0, agg, eta)
                assert (g[: 8 + woff] == 5.0).all() and (g[8 + woff + d:] == 5.0).all()
                if with_bits:
                    assert np.array_equal(bits.cpu().numpy().view(np.uint8)[: (d + 7) // 8],
                                          O.pack_bits(agg))
        finally:
            B.brace_reset_tuning()


def test_update_chunk_by_chunk_equals_whole():
    n, d, eta = 10, 100_003, 0.25
    upd = matrix(n, d, seed=8)
    w0 = torch.randn(d, device=DEV)
    whole = w0.clone()
    B.brace_aggregate_update(upd, 2, whole, eta, 1.0)
    parts = w0.clone()
    for c in range(n):
        B.brace_aggregate_update(upd, 2, parts, eta, 1.0, chunk=c)
    torch.cuda.synchronize()
    assert torch.equal(whole, parts)
    agg = O.brace_direct(upd.cpu().numpy(), 1.0).out
    check_update(whole.cpu().numpy(), w0.cpu().numpy(), agg, eta)
    # the paper's update moves every coordinate by exactly eta (eta = 0.25 is exact in fp32)
    assert torch.equal((whole - w0).abs(), torch.full_like(w0, eta)) or \
        float(((whole - w0).abs() - eta).abs().max()) < 1e-6


@pytest.mark.parametrize("d,off", [(0, 0), (1, 0), (31, 0), (1023, 0), (1024, 0), (1025, 0),
                                   (5000, 0), (70_001, 0), (4096, 1), (10_000, 2)])
def test_expand_and_apply_bits(d, off):
    rng = np.random.default_rng(d + off)
    agg = rng.choice(np.array([-1.0, 1.0], dtype=np.float32), size=d)
    packed = O.pack_bits(agg)
    words = np.zeros(4 * ((d + 31) // 32), dtype=np.uint8)
    words[: packed.shape[0]] = packed
    bits = torch.from_numpy(words.view(np.int32).copy()).to(DEV) if d else torch.empty(0, device=DEV, dtype=torch.int32)
    guard = torch.full((d + 16 + off,), 5.0, device=DEV, dtype=torch.float32)
    out = guard[8 + off: 8 + off + d]
    B.brace_expand_bits(bits, d, out)
    torch.cuda.synchronize()
    g = guard.cpu().numpy()
    assert np.array_equal(g[8 + off: 8 + off + d], agg)
    assert (g[: 8 + off] == 5.0).all() and (g[8 + off + d:] == 5.0).all()
    w0 = rng.standard_normal(d).astype(np.float32)
    out.copy_(torch.from_numpy(w0))
    B.brace_apply_bits(bits, d, 0.03, out)
    torch.cuda.synchronize()
    g = guard.cpu().numpy()
    if d:
        check_update(g[8 + off: 8 + off + d], w0, agg, 0.03)
    assert (g[: 8 + off] == 5.0).all() and (g[8 + off + d:] == 5.0).all()


def test_vote_then_apply_equals_fused():
    # Share-Only as the paper runs it: the owner publishes bits, every client applies them.
    w = synth.WORKLOADS[1]
    upd = synth.generate(w, DEV)
    bits = torch.empty((w.d + 31) // 32, device=DEV, dtype=torch.int32)
    B.brace_aggregate(upd, w.f, 5.0, out=None, out_bits=bits)
    model = torch.randn(w.d, device=DEV, generator=torch.Generator(DEV).manual_seed(3))
    a = model.clone()
    B.brace_apply_bits(bits, w.d, 0.1, a)
    b = model.clone()
    B.brace_aggregate_update(upd, w.f, b, 0.1, 5.0)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


@pytest.mark.parametrize("idx,col_tile,with_bits", [(2, 2_000_000, True), (3, 2_000_000, True),
                                                    (3, 2_000_000, False), (4, 4_000_000, True)])
def test_large_workloads_full(idx, col_tile, with_bits):
    w = synth.WORKLOADS[idx]
    upd = synth.generate(w, DEV)
    model0 = torch.randn(w.d, device=DEV, generator=torch.Generator(DEV).manual_seed(idx))
    model = model0.clone()
    bits = torch.empty((w.d + 31) // 32, device=DEV, dtype=torch.int32) if with_bits else None
    eta = 0.01
    B.brace_aggregate_update(upd, w.f, model, eta, 5.0, out_bits=bits)
    torch.cuda.synchronize()
    got = model.cpu().numpy()
    w0 = model0.cpu().numpy()
    for k0 in range(0, w.d, col_tile):
        k1 = min(w.d, k0 + col_tile)
        host = upd[:, k0:k1].contiguous().cpu().numpy()
        agg, _, _ = C.brace_direct(host, 5.0, 0, want_sums=False, want_bits=False)
        check_update(got[k0:k1], w0[k0:k1], agg, eta)
        print(f"{w.name}: update over columns [{k0}, {k1}) matches", flush=True)
    del upd
    torch.cuda.empty_cache()
