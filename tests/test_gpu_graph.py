"""The entry points allocate nothing and record no memset, so they can be captured in a HIP
graph.  Each graph is replayed several times, with eager work and synchronisations between
the replays and with the input changed in place, and every replay is checked against the CPU
oracle (not only against the eager run)."""

import numpy as np
import pytest
import torch

from oracle import brace_oracle as O
from paper_2501_17392_amd import binding as B

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def fill(upd, seed):
    g = torch.Generator(DEV).manual_seed(seed)
    upd.copy_(torch.randn(upd.shape, device=DEV, generator=g))
    upd[:, ::7] = 0.0


def test_chunk_loop_and_whole_call_in_a_graph():
    assert torch.cuda.is_available()
    B.lib()
    B.brace_reset_tuning()
    n, d, f, lam = 20, 300_007, 4, 2.0
    upd = torch.empty(n, d, device=DEV)
    fill(upd, 0)
    out_chunks = torch.zeros(d, device=DEV)
    out_whole = torch.zeros(d, device=DEV)
    bits = torch.zeros((d + 31) // 32, device=DEV, dtype=torch.int32)
    mean = torch.zeros(d, device=DEV)
    model = torch.zeros(d, device=DEV)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        # warm-up outside the capture (first launches load the code objects)
        B.brace_aggregate(upd, f, lam, out=out_whole, out_bits=bits)
        B.brace_rar_aggregate(upd, mean, mean=True)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            for c in range(n):
                B.brace_aggregate_chunk(upd, f, c, lam, out=out_chunks)
            B.brace_aggregate(upd, f, lam, out=out_whole, out_bits=bits)
            B.brace_rar_aggregate(upd, mean, mean=True)
            B.brace_apply_bits(bits, d, 0.5, model)
    torch.cuda.synchronize()

    applied = np.zeros(d, dtype=np.float64)
    for replay in range(4):
        fill(upd, 100 + replay)                       # eager work between replays
        out_chunks.fill_(7.0)
        out_whole.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        host = upd.cpu().numpy()
        want = O.brace_direct(host, lam)
        assert np.array_equal(out_chunks.cpu().numpy(), want.out), replay
        assert np.array_equal(out_whole.cpu().numpy(), want.out), replay
        assert np.array_equal(bits.cpu().numpy().view(np.uint8)[: (d + 7) // 8], want.bits), replay
        got_mean = mean.cpu().numpy().astype(np.float64)
        ref_mean = O.mean_direct(host)
        assert np.all(np.abs(got_mean - ref_mean) <= 1e-6 + 1e-5 * np.abs(ref_mean)), replay
        applied = O.model_update(applied.astype(np.float32), want.out, 0.5)
        assert np.allclose(model.cpu().numpy(), applied, rtol=1e-5, atol=1e-6), replay
        # an eager call in between gives the same thing
        eager = torch.zeros(d, device=DEV)
        B.brace_aggregate(upd, f, lam, out=eager)
        torch.cuda.synchronize()
        assert torch.equal(eager, out_whole)


def test_planes_route_in_a_graph_after_init_device():
    """Quantise once, vote per run of chunks on the planes, Phase III on partial sums, burst-writing
    sum: captured with only brace_init_device() before (no warm-up launches), replayed and checked
    against the oracle each time.  Rows are long enough for the burst kernels (128 spans, >= 8
    rounds of blocks is forced through the tuning)."""
    assert torch.cuda.is_available()
    B.lib()
    B.brace_reset_tuning()
    n, d, lam = 6, 128 * 4096 * 2 + 4097, 1.0
    upd = torch.empty(n, d, device=DEV)
    fill(upd, 1)
    signs = torch.zeros(n, B.brace_packed_row_words(d), device=DEV, dtype=torch.int32)
    out = torch.zeros(d, device=DEV)
    bits = torch.zeros((d + 31) // 32, device=DEV, dtype=torch.int32)
    parts = torch.zeros(2, d, device=DEV, dtype=torch.int16)
    out3 = torch.zeros(d, device=DEV)
    total = torch.zeros(d, device=DEV)

    B.brace_init_device()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    try:
        B.brace_set_tuning(stage_writes=2)
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                B.brace_quantize(upd, signs)
                bits.zero_()                      # a fill kernel, not a memset node
                B.brace_vote_packed_chunks(signs, d, 0, 0, 2, lam, out=out, out_bits=bits)
                B.brace_vote_packed_chunks(signs, d, 0, 2, n, lam, out=out, out_bits=bits)
                B.brace_aggregate(upd[:3], 0, 0.0, sums=parts[0])
                B.brace_aggregate(upd[3:], 0, 0.0, sums=parts[1])
                B.brace_consensus_sums(parts, lam, out=out3)
                B.brace_rar_aggregate(upd, total)
    finally:
        B.brace_reset_tuning()
    torch.cuda.synchronize()

    for replay in range(3):
        fill(upd, 200 + replay)
        out.fill_(7.0)
        out3.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        host = upd.cpu().numpy()
        want = O.brace_direct(host, lam)
        assert np.array_equal(signs.cpu().numpy().view(np.uint32), O.sign_planes(host)), replay
        assert np.array_equal(out.cpu().numpy(), want.out), replay
        assert np.array_equal(out3.cpu().numpy(), want.out), replay
        assert np.array_equal(bits.cpu().numpy().view(np.uint8)[: (d + 7) // 8], want.bits), replay
        ref = O.rar_sum_direct(host)
        got = total.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - ref) <= 1e-6 + 1e-5 * np.abs(ref)), replay


def test_noalloc_update_ring_order_and_wide_quantize_in_a_graph():
    """The allocation-free fused update (its bit-words live in the library's own workspace, whose
    address brace_init_device looks up ahead of the capture), the ring-order fp32 sum and the
    4-dword burst quantize, captured without warm-up launches and replayed with new inputs."""
    assert torch.cuda.is_available()
    B.lib()
    B.brace_reset_tuning()
    n, d, lam, eta = 12, 144 * 4096 + 8192 + 4, 1.0, 0.25        # rows of whole 16-byte vectors
    upd = torch.empty(n, d, device=DEV)
    fill(upd, 3)
    w = torch.zeros(d, device=DEV)
    total = torch.zeros(d, device=DEV)
    rw, rp = B.brace_packed_row_words(d), B.brace_packed_row_pitch(d)
    signs = torch.zeros(n, rp, device=DEV, dtype=torch.int32)[:, :rw]
    vw, vp = B.brace_1bit_row_words(d), B.brace_1bit_row_pitch(d)
    votes = torch.zeros(n, vp, device=DEV, dtype=torch.int32)[:, :vw]
    out = torch.zeros(d, device=DEV)

    B.brace_init_device()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    try:
        B.brace_set_tuning(split_writes=2, stage_writes=2)
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                B.brace_aggregate_update_noalloc(upd, 0, w, eta, lam)
                B.brace_rar_aggregate(upd, total, order=1)
                B.brace_quantize(upd, signs)
                B.brace_quantize_1bit(upd, -1, votes)
                B.brace_vote_1bit(votes, d, 0, lam, out=out)
    finally:
        B.brace_reset_tuning()
    torch.cuda.synchronize()

    model = np.zeros(d, dtype=np.float32)
    for replay in range(3):
        fill(upd, 300 + replay)
        out.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        host = upd.cpu().numpy()
        want = O.brace_direct(host, lam)
        model = O.model_update(model, want.out, np.float32(eta)).astype(np.float32)
        assert np.array_equal(w.cpu().numpy(), model), replay          # +-0.25 steps are exact in fp32
        ring = O.rar_sum_ring_order(host)
        assert np.array_equal(total.cpu().numpy().view(np.uint32), ring.view(np.uint32)), replay
        assert np.array_equal(signs.cpu().numpy().view(np.uint32), O.sign_planes(host)), replay
        assert np.array_equal(votes.cpu().numpy().view(np.uint32), O.vote_plane(host, -1)), replay
        assert np.array_equal(out.cpu().numpy(), O.brace_direct(host, lam, -1).out), replay
        # the same entry point called eagerly in between gives the same model
        w2 = torch.from_numpy(model).to(DEV)
        w3 = w2.clone()
        B.brace_aggregate_update_noalloc(upd, 0, w2, eta, lam)
        B.brace_aggregate_update(upd, 0, w3, eta, lam)
        torch.cuda.synchronize()
        assert torch.equal(w2, w3)
