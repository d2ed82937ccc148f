"""More than 2^31 coordinates in one vector: every coordinate index in the kernels and in the
host planning is 64-bit, and this is the case that shows it.  n = 2 clients, d = 2^31 + 4099
(17 GB of input).  The oracle checks windows of 4 M coordinates at the start, across the 2^31
boundary, at the ragged end and at seeded random places; everywhere else the output is checked
for the properties that hold at any size (values in {-1, +1}, bits equal to the floats)."""

import numpy as np
import pytest
import torch

from oracle import brace_oracle as O
from oracle import c_oracle as C
from paper_2501_17392_amd import binding as B

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
D = (1 << 31) + 4099
WIN = 1 << 22


def windows():
    rng = np.random.default_rng(31)
    starts = [0, (1 << 31) - WIN // 2, D - WIN]
    starts += [int(x) for x in rng.integers(0, D - WIN, size=4)]
    return [(s, min(D, s + WIN)) for s in starts]


def test_vector_longer_than_2_to_31():
    assert torch.cuda.is_available()
    B.lib()
    B.brace_reset_tuning()
    n, lam = 2, 0.0
    upd = torch.empty(n, D, device=DEV, dtype=torch.float32)
    gen = torch.Generator(DEV).manual_seed(2031)
    step = 1 << 28
    for k in range(0, D, step):                      # filled in pieces: no 17 GB temporary
        upd[:, k: k + step].normal_(generator=gen)
    upd[:, ::5] = 0.0
    out = torch.empty(D, device=DEV, dtype=torch.float32)
    bits = torch.empty((D + 31) // 32, device=DEV, dtype=torch.int32)
    sums = torch.empty(D, device=DEV, dtype=torch.int16)
    B.brace_aggregate(upd, 0, lam, out=out, out_bits=bits, sums=sums)
    torch.cuda.synchronize()
    print("vote done", flush=True)

    # properties over the whole vector, on the device
    assert bool(((out == 1.0) | (out == -1.0)).all())
    assert bool(((sums > lam) == (out > 0)).all())
    nwords = D // 32
    for k in range(0, nwords, 1 << 24):              # bits == floats, 2^29 coordinates at a time
        w = bits[k: min(k + (1 << 24), nwords)]
        seg = (out[32 * k: 32 * (k + w.numel())] > 0).view(-1, 32)
        packed = (seg.to(torch.int64) << torch.arange(32, device=DEV)).sum(dim=1)
        assert torch.equal(packed, w.to(torch.int64) & 0xFFFFFFFF), k
    print("properties hold", flush=True)

    # the oracle on windows
    for lo, hi in windows():
        host = upd[:, lo:hi].contiguous().cpu().numpy()
        want, want_sums, _ = C.brace_direct(host, lam, 0, want_sums=True, want_bits=False)
        assert np.array_equal(out[lo:hi].cpu().numpy(), want), (lo, hi)
        assert np.array_equal(sums[lo:hi].cpu().numpy().astype(np.int64), want_sums.astype(np.int64)), (lo, hi)
        print(f"window [{lo}, {hi}) matches", flush=True)
    tail = bits[-1:].cpu().numpy().view(np.uint32)[0]
    assert tail >> (D % 32) == 0, "padding bits of the last word must be zero"
    del sums

    # the same vector through the planes, per run of chunks, and the plain sum
    signs = torch.empty(n, B.brace_packed_row_words(D), device=DEV, dtype=torch.int32)
    B.brace_quantize(upd, signs)
    out2 = torch.empty(D, device=DEV, dtype=torch.float32)
    B.brace_vote_packed_chunks(signs, D, 0, 0, 1, lam, out=out2)
    B.brace_vote_packed_chunks(signs, D, 0, 1, 2, lam, out=out2)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    del out2, signs
    total = torch.empty(D, device=DEV, dtype=torch.float32)
    B.brace_rar_aggregate(upd, total)
    torch.cuda.synchronize()
    for lo, hi in windows()[:3]:
        host = upd[:, lo:hi].contiguous().cpu().numpy()
        ref = O.rar_sum_direct(host)
        got = total[lo:hi].cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - ref) <= 1e-6 + 1e-5 * np.abs(ref)), (lo, hi)
    print("planes route and sum match", flush=True)
    del upd, out, bits, total
    torch.cuda.empty_cache()
