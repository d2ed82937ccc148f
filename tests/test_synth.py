"""The seeded input generators: shapes, determinism and the structure each workload promises."""

import numpy as np
import torch

from paper_2501_17392_amd import synth


def test_workload_table_matches_the_benchmark_configs():
    got = [(w.n, w.f, w.d, w.seed) for w in synth.WORKLOADS]
    assert got == [(10, 2, 10_000, 0), (20, 4, 1_000_003, 1), (50, 10, 11_173_962, 2),
                   (100, 20, 25_000_000, 3), (64, 16, 100_000_000, 4)]
    assert synth.WORKLOADS[3].input_bytes == 10_000_000_000


def test_generate_is_deterministic_and_tile_addressable():
    w = synth.WORKLOADS[1].with_d(synth.TILE + 1234)
    a = synth.generate(w, "cpu")
    b = synth.generate(w, "cpu")
    assert a.shape == (w.n, w.d) and a.dtype == torch.float32
    assert torch.equal(a, b)
    t1 = synth.generate_tile(w, 1, "cpu")
    assert t1.shape == (w.n, 1234)
    assert torch.equal(a[:, synth.TILE:], t1)
    assert synth.checksum(a) == synth.checksum(b)


def test_pitched_allocation_pads_with_nan():
    w = synth.WORKLOADS[0].with_d(1001)
    v = synth.generate(w, "cpu", ld=1024)
    assert v.shape == (w.n, 1001) and v.stride(0) == 1024
    dense = synth.generate(w, "cpu")
    assert torch.equal(v, dense)


def test_cfg0_signflip_rows():
    w = synth.WORKLOADS[0]
    g = synth.generate(w, "cpu")
    nb = w.n - w.f
    mean_b = g[:nb].mean(dim=0)
    for r in range(nb, w.n):
        assert torch.equal(g[r], -3.0 * mean_b)
    assert abs(float(g[:nb].std()) - 0.1) < 0.01


def test_cfg1_gaussian_attack_scale():
    w = synth.WORKLOADS[1].with_d(50_000)
    g = synth.generate(w, "cpu")
    assert 150 < float(g[w.n - w.f:].std()) < 250


def test_cfg2_heterogeneous_scales_and_inversion():
    w = synth.WORKLOADS[2].with_d(40_000)
    g = synth.generate(w, "cpu")
    s = synth.client_scales(w)
    assert float(s.min()) >= 0.05 and float(s.max()) <= 0.3
    stds = g[: w.n - w.f].std(dim=1)
    assert torch.allclose(stds, s[: w.n - w.f], rtol=0.05)
    byz_std = g[w.n - w.f:].std(dim=1)
    assert torch.allclose(byz_std, 10.0 * s[w.n - w.f:], rtol=0.05)


def test_cfg3_little_is_enough_rows_are_identical_and_inside_the_benign_spread():
    w = synth.WORKLOADS[3].with_d(20_000)
    g = synth.generate(w, "cpu")
    nb = w.n - w.f
    for r in range(nb + 1, w.n):
        assert torch.equal(g[r], g[nb])
    b = g[:nb]
    want = b.mean(0) - 1.5 * b.std(0, unbiased=False)
    assert torch.allclose(g[nb], want, rtol=1e-5, atol=1e-6)
    # heavy tails: Student-t(3) has far more 6-sigma draws than a normal
    z = (b - b.mean()) / 0.1
    assert int((z.abs() > 6).sum()) > 50


def test_cfg4_exact_zeros_and_negative_zero():
    w = synth.WORKLOADS[4].with_d(100_000)
    g = synth.generate(w, "cpu")
    nb = w.n - w.f
    zero_cols = (g[:nb] == 0).all(dim=0)
    frac = float(zero_cols.float().mean())
    assert 0.005 < frac < 0.02
    assert not ((g[:nb] == 0).any(dim=0) & ~zero_cols).any()
    flip = g[nb: nb + w.f // 2]
    assert (flip[:, zero_cols] == 0).all()
    assert torch.signbit(flip[:, zero_cols]).all()          # -3 * (+0) = -0.0
    noise = g[nb + w.f // 2:]
    assert 150 < float(noise.std()) < 250
