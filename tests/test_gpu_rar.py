"""GPU parity for the plain ring-all-reduce sum / mean (the operation BRACE replaces, Sec. 2.2
and Sec. 2.1) against the fp64 CPU oracle.

Tolerance: |gpu - oracle| <= 1e-6 + 1e-5 * |oracle| (the bar stated for floating-point sums).
The kernel accumulates in fp64 and rounds to fp32 once, so the expected error is one fp32
rounding (6e-8 relative) whatever the cancellation between rows.
"""

import json
import os

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


def close(got, want):
    got = np.asarray(got, dtype=np.float64)
    return np.all(np.abs(got - want) <= ATOL + RTOL * np.abs(want))


def device_matrix(n, d, seed, ld=None, offset=0, scale=1.0):
    rng = np.random.default_rng(seed)
    g = (scale * rng.standard_normal((n, d))).astype(np.float32)
    g[rng.random((n, d)) < 0.05] = 0.0
    ld = d if ld is None else ld
    store = torch.full((n * max(ld, 1) + offset + 8,), float("nan"), device=DEV, dtype=torch.float32)
    view = store[offset: offset + n * max(ld, 1)].view(n, max(ld, 1))[:, :d]
    view.copy_(torch.from_numpy(g))
    return view


def test_three_client_example_through_the_gpu(golden_dir):
    # Sec. 2.2 example and its attacked variant from Sec. 3, exact in fp32.
    with open(os.path.join(golden_dir, "rar_three_client_example.json")) as fh:
        ex = json.load(fh)
    g = torch.tensor(ex["gradients"], device=DEV, dtype=torch.float32)
    out = torch.empty(3, device=DEV, dtype=torch.float32)
    B.brace_rar_aggregate(g, out)
    torch.cuda.synchronize()
    assert out.cpu().tolist() == [22.0, 1.0, 5.0]
    g[0] = torch.tensor(ex["attacked_gradient_client1"], device=DEV, dtype=torch.float32)
    B.brace_rar_aggregate(g, out)
    torch.cuda.synchronize()
    assert out.cpu().tolist() == [float(v) for v in ex["attacked_aggregate"]]
    for c in range(3):          # one chunk per client, as in the example
        piece = torch.full((3,), 99.0, device=DEV, dtype=torch.float32)
        B.brace_rar_aggregate(g, piece, chunk=c)
        torch.cuda.synchronize()
        want = [99.0] * 3
        want[c] = float(ex["attacked_aggregate"][c])
        assert piece.cpu().tolist() == want


@pytest.mark.parametrize("n,d,ld,offset", [
    (1, 1, None, 0), (2, 5, None, 0), (3, 64, None, 0), (5, 257, None, 0), (7, 1000, None, 0),
    (10, 4099, None, 0), (33, 70_001, None, 0), (100, 20_000, None, 0), (8, 5000, 5004, 0),
    (8, 5000, 5002, 0), (8, 5000, 5001, 0), (9, 12_345, None, 1), (9, 12_345, None, 2),
    (9, 12_344, None, 3), (20, 50_003, None, 0)])
def test_sum_and_mean_small_shapes(n, d, ld, offset):
    upd = device_matrix(n, d, seed=n * 7 + d, ld=ld, offset=offset)
    host = upd.cpu().numpy()
    out = torch.full((d,), 7.0, device=DEV, dtype=torch.float32)
    B.brace_rar_aggregate(upd, out)
    torch.cuda.synchronize()
    assert close(out.cpu().numpy(), O.rar_sum_direct(host))
    B.brace_rar_aggregate(upd, out, mean=True)
    torch.cuda.synchronize()
    assert close(out.cpu().numpy(), O.mean_direct(host))


def test_heavy_cancellation_needs_the_fp64_accumulator():
    # Rows of +-1e6 that cancel to O(1): an fp32 running sum would miss the tolerance.
    n, d = 64, 30_000
    rng = np.random.default_rng(4)
    big = (1e6 * rng.standard_normal((n // 2, d))).astype(np.float32)
    small = rng.standard_normal((1, d)).astype(np.float32)
    g = np.vstack([big, -big[::-1], small, -small * 0.5])[: n]
    upd = torch.from_numpy(np.ascontiguousarray(g)).to(DEV)
    out = torch.empty(d, device=DEV, dtype=torch.float32)
    B.brace_rar_aggregate(upd, out)
    torch.cuda.synchronize()
    want = O.rar_sum_direct(g)
    assert close(out.cpu().numpy(), want)
    fp32_running = np.zeros(d, dtype=np.float32)
    for i in range(g.shape[0]):
        fp32_running += g[i]
    assert not close(fp32_running, want)        # the tolerance really is out of fp32's reach here


def test_non_finite_values_propagate():
    g = torch.tensor([[1.0, float("inf"), float("nan"), float("inf")],
                      [2.0, 1.0, 1.0, float("-inf")]], device=DEV)
    out = torch.empty(4, device=DEV)
    B.brace_rar_aggregate(g, out)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert o[0] == 3.0 and o[1] == np.inf and np.isnan(o[2]) and np.isnan(o[3])


@pytest.mark.parametrize("n,d", [(3, 3), (7, 3), (10, 10_000), (20, 100_003), (13, 4096)])
def test_chunks_tile_the_whole(n, d):
    upd = device_matrix(n, d, seed=n + d)
    whole = torch.empty(d, device=DEV, dtype=torch.float32)
    B.brace_rar_aggregate(upd, whole, mean=True)
    parts = torch.full((d,), 7.0, device=DEV, dtype=torch.float32)
    for c in range(n):
        B.brace_rar_aggregate(upd, parts, mean=True, chunk=c)
    torch.cuda.synchronize()
    assert torch.equal(whole, parts)
    assert close(whole.cpu().numpy(), O.mean_direct(upd.cpu().numpy()))


def test_tunings_agree():
    n, d = 19, 200_003
    upd = device_matrix(n, d, seed=1, ld=d + 1)
    want = O.rar_sum_direct(upd.cpu().numpy())
    ref = None
    try:
        for vec in (0, 1, 2, 4):
            for cols in (1, 2, 4, 8):
                for unroll in (2, 4, 8):
                    for nt, pipe, rs in ((0, 0, 1), (1, 1, 1), (1, 1, 2), (0, 0, 2)):
                        B.brace_set_tuning(vec, cols, unroll, nt, pipe, 0, rs)
                        out = torch.empty(d, device=DEV, dtype=torch.float32)
                        B.brace_rar_aggregate(upd, out)
                        torch.cuda.synchronize()
                        got = out.cpu().numpy()
                        assert close(got, want), (vec, cols, unroll, nt, pipe, rs)
                        if rs == 1:
                            if ref is None:
                                ref = got
                            # same row order without the row split -> bitwise identical
                            assert np.array_equal(got, ref)
    finally:
        B.brace_reset_tuning()


@pytest.mark.parametrize("idx", [0, 1])
def test_small_workloads_full(idx):
    w = synth.WORKLOADS[idx]
    upd = synth.generate(w, DEV)
    host = upd.cpu().numpy()
    out = torch.empty(w.d, device=DEV, dtype=torch.float32)
    B.brace_rar_aggregate(upd, out)
    torch.cuda.synchronize()
    assert close(out.cpu().numpy(), O.rar_sum_direct(host))
    if idx == 0:
        ring = O.ring_all_reduce(host, mode="sum")
        for b in ring.buffers:
            assert close(out.cpu().numpy(), b)


@pytest.mark.parametrize("idx,col_tile", [(2, 2_000_000), (3, 2_000_000), (4, 4_000_000)])
def test_large_workloads_full(idx, col_tile):
    w = synth.WORKLOADS[idx]
    upd = synth.generate(w, DEV)
    out = torch.empty(w.d, device=DEV, dtype=torch.float32)
    B.brace_rar_aggregate(upd, out, mean=True)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for k0 in range(0, w.d, col_tile):
        k1 = min(w.d, k0 + col_tile)
        host = upd[:, k0:k1].contiguous().cpu().numpy()
        want = C.rar_sum(host, 1.0 / w.n)
        assert close(got[k0:k1], want), (w.name, k0)
        print(f"{w.name}: mean over columns [{k0}, {k1}) matches", flush=True)
    del upd
    torch.cuda.empty_cache()


@pytest.mark.parametrize("n,d,ld,offset", [(3, 64, None, 0), (5, 257, None, 0), (7, 8192, None, 0),
                                           (7, 8193, None, 0), (10, 40_000, None, 0),
                                           (33, 70_001, None, 0), (8, 50_000, 50_002, 0),
                                           (8, 50_000, 50_001, 0), (9, 123_456, None, 2),
                                           (20, 300_007, None, 0)])
def test_staged_burst_writes_forced(n, d, ld, offset):
    # The LDS-staged kernel (one contiguous burst per block) forced on small and ragged inputs.
    upd = device_matrix(n, d, seed=n * 3 + d, ld=ld, offset=offset)
    host = upd.cpu().numpy()
    try:
        B.brace_set_tuning(stage_writes=2)
        guard = torch.full((d + 64,), 3.0, device=DEV, dtype=torch.float32)
        out = guard[32: 32 + d]
        B.brace_rar_aggregate(upd, out)
        torch.cuda.synchronize()
        g = guard.cpu().numpy()
        assert close(g[32: 32 + d], O.rar_sum_direct(host))
        assert (g[:32] == 3.0).all() and (g[32 + d:] == 3.0).all()
        B.brace_set_tuning(stage_writes=1)
        ref = torch.empty(d, device=DEV, dtype=torch.float32)
        B.brace_rar_aggregate(upd, ref)
        torch.cuda.synchronize()
        assert np.array_equal(ref.cpu().numpy(), g[32: 32 + d])     # same row order: bitwise equal
        parts = torch.full((d,), 7.0, device=DEV, dtype=torch.float32)
        B.brace_set_tuning(stage_writes=2)
        for c in range(n):
            B.brace_rar_aggregate(upd, parts, chunk=c)
        torch.cuda.synchronize()
        assert np.array_equal(parts.cpu().numpy(), g[32: 32 + d])
    finally:
        B.brace_reset_tuning()
