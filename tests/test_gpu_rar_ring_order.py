"""GPU parity for the plain ring-all-reduce sum as a ring of fp32 clients delivers it
(Sec. 2.2 Share-Reduce: ring chunk c is accumulated in the order c, c+1, ..., c-1 (mod n), one
fp32 rounding per addition) -- `order = 1` of brace_rar_aggregate.

Every addition is the same IEEE operation on both sides in the same order, so the bar is
BIT-EXACT against the oracle's fp32 ring (numpy per chunk, the message-by-message ring on small
inputs, the plain-C loop at full size).  Against the exact (fp64) sum the result obeys the
forward error bound of recursive summation, (n - 1) * 2^-24 * sum_i |g_i[k]|; it is NOT inside
1e-6 + 1e-5 |sum| everywhere (large Byzantine rows that cancel), which is why order 0 (fp64
accumulation) is the library's default.
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


@pytest.fixture(scope="module", autouse=True)
def _gpu_and_library():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    B.lib()
    B.brace_reset_tuning()
    yield
    B.brace_reset_tuning()


def bits_equal(got, want):
    got = np.ascontiguousarray(got, dtype=np.float32)
    want = np.ascontiguousarray(want, dtype=np.float32)
    same = got.view(np.uint32) == want.view(np.uint32)
    return bool((same | (np.isnan(got) & np.isnan(want))).all())


def device_matrix(n, d, seed, ld=None, offset=0):
    rng = np.random.default_rng(seed)
    # magnitudes spread over seven decades per client: every addition rounds
    g = (rng.standard_normal((n, d)) * 10.0 ** rng.integers(-3, 4, size=(n, 1))).astype(np.float32)
    g[rng.random((n, d)) < 0.03] = 0.0
    g[rng.random((n, d)) < 0.01] = -0.0
    ld = d if ld is None else ld
    store = torch.full((n * max(ld, 1) + offset + 8,), float("nan"), device=DEV, dtype=torch.float32)
    view = store[offset: offset + n * max(ld, 1)].view(n, max(ld, 1))[:, :d]
    view.copy_(torch.from_numpy(g))
    return view


def test_printed_example_and_the_order_pin_through_the_gpu(golden_dir):
    with open(os.path.join(golden_dir, "rar_three_client_example.json")) as fh:
        ex = json.load(fh)
    g = torch.tensor(ex["gradients"], device=DEV, dtype=torch.float32)
    out = torch.empty(3, device=DEV, dtype=torch.float32)
    B.brace_rar_aggregate(g, out, order=1)
    torch.cuda.synchronize()
    assert out.cpu().tolist() == [22.0, 1.0, 5.0]
    g[0] = torch.tensor(ex["attacked_gradient_client1"], device=DEV, dtype=torch.float32)
    B.brace_rar_aggregate(g, out, order=1)
    torch.cuda.synchronize()
    assert out.cpu().tolist() == [float(v) for v in ex["attacked_aggregate"]]
    # (2^24, 1, 1) in every coordinate: chunk 1 adds 1 + 1 first and keeps the 2, chunks 0 and
    # 2 lose both ones to rounding -- the order c, c+1, ... shows in the bits.
    big = float(2 ** 24)
    g = torch.tensor([[big] * 6, [1.0] * 6, [1.0] * 6], device=DEV, dtype=torch.float32)
    out = torch.empty(6, device=DEV, dtype=torch.float32)
    B.brace_rar_aggregate(g, out, order=1)
    torch.cuda.synchronize()
    assert out.cpu().tolist() == [big, big, big + 2, big + 2, big, big]
    B.brace_rar_aggregate(g, out, order=0)                  # fp64 accumulation: the exact sum
    torch.cuda.synchronize()
    assert out.cpu().tolist() == [big + 2] * 6


@pytest.mark.parametrize("n,d,ld,offset", [
    (1, 1, None, 0), (1, 700, None, 0), (2, 5, None, 0), (3, 3, None, 0), (7, 3, None, 0),
    (3, 64, None, 0), (5, 257, None, 0), (7, 1000, None, 0), (10, 4099, None, 0),
    (4, 2048, None, 0), (4, 2049, None, 0), (2, 1023, None, 0), (3, 1536, None, 0),
    (33, 70_001, None, 0), (100, 20_000, None, 0), (8, 5000, 5004, 0), (8, 5000, 5002, 0),
    (8, 5000, 5001, 0), (9, 12_345, None, 1), (9, 12_345, None, 2), (9, 12_344, None, 3),
    (20, 50_003, None, 0), (6, 400_000, None, 0), (3, 1_000_001, None, 0), (64, 70, None, 0)])
def test_ring_order_sum_and_mean_bit_exact(n, d, ld, offset):
    upd = device_matrix(n, d, seed=n * 11 + d, ld=ld, offset=offset)
    host = upd.cpu().numpy()
    guard = torch.full((d + 64,), 3.0, device=DEV, dtype=torch.float32)
    out = guard[32: 32 + d]
    B.brace_rar_aggregate(upd, out, order=1)
    torch.cuda.synchronize()
    g = guard.cpu().numpy()
    want = O.rar_sum_ring_order(host)
    assert bits_equal(g[32: 32 + d], want)
    assert (g[:32] == 3.0).all() and (g[32 + d:] == 3.0).all()
    if n * d <= 200_000:                                    # the literal ring, message by message
        for b in O.ring_all_reduce(host, mode="sum", dtype=np.float32).buffers:
            assert bits_equal(g[32: 32 + d], b)
    B.brace_rar_aggregate(upd, out, mean=True, order=1)
    torch.cuda.synchronize()
    assert bits_equal(out.cpu().numpy(), O.mean_ring_order(host))
    # against the exact sum: the forward error bound of recursive summation in fp32
    exact = O.rar_sum_direct(host)
    bound = (n - 1) * 2.0 ** -24 * np.abs(host.astype(np.float64)).sum(axis=0) * 1.01 + 1e-45
    assert (np.abs(g[32: 32 + d].astype(np.float64) - exact) <= bound).all()


@pytest.mark.parametrize("n,d", [(3, 3), (7, 3), (10, 10_000), (20, 100_003), (13, 4096), (5, 1_000_003)])
def test_ring_order_chunks_tile_the_whole(n, d):
    upd = device_matrix(n, d, seed=n + d)
    whole = torch.empty(d, device=DEV, dtype=torch.float32)
    B.brace_rar_aggregate(upd, whole, order=1)
    parts = torch.full((d,), 7.0, device=DEV, dtype=torch.float32)
    for c in range(n):
        before = parts.clone()
        B.brace_rar_aggregate(upd, parts, chunk=c, order=1)
        torch.cuda.synchronize()
        lo, hi = O.chunk_range(n, d, c)
        assert torch.equal(parts[:lo], before[:lo]) and torch.equal(parts[hi:], before[hi:])
    assert bits_equal(parts.cpu().numpy(), whole.cpu().numpy())
    assert bits_equal(whole.cpu().numpy(), O.rar_sum_ring_order(upd.cpu().numpy()))


def test_ring_order_load_widths_and_tile_shapes_agree():
    n, d = 19, 200_003
    upd = device_matrix(n, d, seed=1, ld=d + 1)
    want = O.rar_sum_ring_order(upd.cpu().numpy())
    try:
        for vec in (0, 1, 2, 4):
            for cols in (0, 1, 2, 4, 8):
                for stage in (0, 1, 2):
                    B.brace_set_tuning(vec=vec, cols=cols, stage_writes=stage)
                    out = torch.empty(d, device=DEV, dtype=torch.float32)
                    B.brace_rar_aggregate(upd, out, order=1)
                    torch.cuda.synchronize()
                    assert bits_equal(out.cpu().numpy(), want), (vec, cols, stage)
    finally:
        B.brace_reset_tuning()


@pytest.mark.parametrize("n,d,ld,offset", [(3, 64, None, 0), (5, 257, None, 0), (7, 8192, None, 0),
                                           (7, 8193, None, 0), (10, 40_000, None, 0),
                                           (33, 70_001, None, 0), (8, 50_000, 50_002, 0),
                                           (8, 50_000, 50_001, 0), (9, 123_456, None, 2),
                                           (20, 300_007, None, 0), (100, 250_000, None, 0),
                                           (300, 70_000, None, 0)])
def test_ring_order_staged_bursts_forced(n, d, ld, offset):
    # The burst-writing variant forced on small and ragged inputs: many chunk boundaries fall
    # inside a wave's run of slots and inside single slots (300 clients x 70,000: chunks of 233).
    upd = device_matrix(n, d, seed=n * 3 + d, ld=ld, offset=offset)
    want = O.rar_sum_ring_order(upd.cpu().numpy())
    try:
        B.brace_set_tuning(stage_writes=2)
        guard = torch.full((d + 64,), 3.0, device=DEV, dtype=torch.float32)
        out = guard[32: 32 + d]
        B.brace_rar_aggregate(upd, out, order=1)
        torch.cuda.synchronize()
        g = guard.cpu().numpy()
        assert bits_equal(g[32: 32 + d], want)
        assert (g[:32] == 3.0).all() and (g[32 + d:] == 3.0).all()
        parts = torch.full((d,), 7.0, device=DEV, dtype=torch.float32)
        for c in range(n):
            B.brace_rar_aggregate(upd, parts, chunk=c, order=1)
        torch.cuda.synchronize()
        assert bits_equal(parts.cpu().numpy(), want)
    finally:
        B.brace_reset_tuning()


def test_non_finite_values_propagate_in_ring_order():
    g = torch.tensor([[1.0, float("inf"), float("nan"), float("inf")],
                      [2.0, 1.0, 1.0, float("-inf")]], device=DEV)
    out = torch.empty(4, device=DEV)
    B.brace_rar_aggregate(g, out, order=1)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert o[0] == 3.0 and o[1] == np.inf and np.isnan(o[2]) and np.isnan(o[3])


@pytest.mark.parametrize("idx", [0, 1])
def test_small_workloads_full_ring_order(idx):
    w = synth.WORKLOADS[idx]
    upd = synth.generate(w, DEV)
    host = upd.cpu().numpy()
    out = torch.empty(w.d, device=DEV, dtype=torch.float32)
    B.brace_rar_aggregate(upd, out, order=1)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert bits_equal(got, O.rar_sum_ring_order(host))
    assert bits_equal(got, C.rar_sum_ring_f32(host))
    if idx == 0:
        for b in O.ring_all_reduce(host, mode="sum", dtype=np.float32).buffers:
            assert bits_equal(got, b)
        # no large rows in this workload: the fp32 ring also meets the float bar here
        exact = O.rar_sum_direct(host)
        assert (np.abs(got.astype(np.float64) - exact) <= 1e-6 + 1e-5 * np.abs(exact)).all()


@pytest.mark.parametrize("idx,col_tile", [(2, 2_000_000), (3, 2_000_000), (4, 4_000_000)])
def test_large_workloads_full_ring_order(idx, col_tile):
    # Full size, the launch bench.py times; the plain-C ring loop streamed in column tiles
    # (it takes the tile's position in the full vector, which decides each column's chunk).
    w = synth.WORKLOADS[idx]
    upd = synth.generate(w, DEV)
    out = torch.empty(w.d, device=DEV, dtype=torch.float32)
    B.brace_rar_aggregate(upd, out, mean=True, order=1)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for k0 in range(0, w.d, col_tile):
        k1 = min(w.d, k0 + col_tile)
        host = upd[:, k0:k1].contiguous().cpu().numpy()
        want = C.rar_sum_ring_f32(host, mean=True, d_total=w.d, k0=k0)
        assert bits_equal(got[k0:k1], want), (w.name, k0)
        print(f"{w.name}: ring-order mean over columns [{k0}, {k1}) bit-exact", flush=True)
    del upd
    torch.cuda.empty_cache()
