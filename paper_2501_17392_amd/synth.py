"""Seeded synthetic client updates for the five benchmark workloads.

This module only draws inputs.  It holds none of the aggregation method's
arithmetic (no sign, no vote, no threshold) and is the one piece of code that
both the HIP path's callers and the CPU oracle's tests use, so that both sides
always see the same bytes.

The workloads stand in for the gradient matrices of the paper's experiments
(Sec. 5.1: n = 100 clients, 20 % malicious); the datasets and models behind
those are not needed because the aggregation cost is independent of the data.

Recipe (per workload; `mu` is one vector shared by all clients):
  benign rows 0 .. n-f-1, Byzantine rows n-f .. n-1.
  gauss     : mu + N(0, 0.1^2),   mu ~ N(0, 0.01^2)
  hetero    : mu + N(0, s_i^2),   s_i ~ U[0.05, 0.3] per client
  student_t : mu + 0.1 * StudentT(df = 3)
  sparse    : gauss, then a shared 1 % coordinate mask set to exactly 0
  attacks   : signflip   -3 * mean_benign
              gaussian   N(0, 200^2)
              inversion  -10 * (a benign draw of that row)
              lie        mean_benign - 1.5 * std_benign (population std)
              mix        first half of the Byzantine rows signflip, rest gaussian
Columns are drawn in fixed tiles of TILE columns, each tile from its own
generator seeded by (seed, tile index), so a tile can be regenerated alone.
"""

from __future__ import annotations

from dataclasses import dataclass, replace

import torch

TILE = 1 << 20


@dataclass(frozen=True)
class Workload:
    name: str
    n: int
    f: int
    d: int
    seed: int
    benign: str
    attack: str

    def with_d(self, d: int) -> "Workload":
        """Same recipe at another dimension (for small parity cases)."""
        return replace(self, d=int(d), name=f"{self.name}@d={int(d)}")

    @property
    def input_bytes(self) -> int:
        return 4 * self.n * self.d


WORKLOADS = (
    Workload("cfg0_n10_d10k_signflip", 10, 2, 10_000, 0, "gauss", "signflip"),
    Workload("cfg1_n20_d1000003_gaussian", 20, 4, 1_000_003, 1, "gauss", "gaussian"),
    Workload("cfg2_n50_d11173962_inversion", 50, 10, 11_173_962, 2, "hetero", "inversion"),
    Workload("cfg3_n100_d25M_lie", 100, 20, 25_000_000, 3, "student_t", "lie"),
    Workload("cfg4_n64_d100M_sparse_mix", 64, 16, 100_000_000, 4, "sparse", "mix"),
)


def _gen(device, seed: int, stream: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) << 32) + int(stream))
    return g


def client_scales(w: Workload) -> torch.Tensor:
    """Per-client noise scale s_i (only 'hetero' differs from 0.1); drawn on the CPU."""
    if w.benign == "hetero":
        g = _gen("cpu", w.seed, (1 << 31) - 1)
        u = torch.rand(w.n, generator=g, dtype=torch.float32)
        return 0.05 + 0.25 * u
    return torch.full((w.n,), 0.1, dtype=torch.float32)


def _noise(w: Workload, rows: int, cols: int, g: torch.Generator, device) -> torch.Tensor:
    """Unit-scale benign noise for `rows` clients."""
    z = torch.randn(rows, cols, generator=g, device=device, dtype=torch.float32)
    if w.benign == "student_t":
        chi = torch.zeros(rows, cols, device=device, dtype=torch.float32)
        for _ in range(3):
            chi += torch.randn(rows, cols, generator=g, device=device, dtype=torch.float32) ** 2
        z = z / torch.sqrt(chi / 3.0)
    return z


def generate_tile(w: Workload, t: int, device) -> torch.Tensor:
    """Columns [t*TILE, min(d, (t+1)*TILE)) of the n x d update matrix, shape (n, width)."""
    lo = t * TILE
    hi = min(w.d, lo + TILE)
    if lo >= hi:
        return torch.empty(w.n, 0, device=device, dtype=torch.float32)
    cols = hi - lo
    nb = w.n - w.f
    g = _gen(device, w.seed, t)
    scales = client_scales(w).to(device)

    mu = 0.01 * torch.randn(1, cols, generator=g, device=device, dtype=torch.float32)
    benign = mu + scales[:nb, None] * _noise(w, nb, cols, g, device)
    if w.benign == "sparse":
        mask = torch.rand(1, cols, generator=g, device=device) < 0.01
        benign = torch.where(mask, torch.zeros((), device=device), benign)

    out = torch.empty(w.n, cols, device=device, dtype=torch.float32)
    out[:nb] = benign
    if w.f == 0:
        return out
    mean_b = benign.mean(dim=0, keepdim=True)

    def signflip(rows):
        return (-3.0 * mean_b).expand(rows, cols)

    def gaussian(rows):
        return 200.0 * torch.randn(rows, cols, generator=g, device=device, dtype=torch.float32)

    if w.attack == "signflip":
        byz = signflip(w.f)
    elif w.attack == "gaussian":
        byz = gaussian(w.f)
    elif w.attack == "inversion":
        own = mu + scales[nb:, None] * _noise(w, w.f, cols, g, device)
        byz = -10.0 * own
    elif w.attack == "lie":
        std_b = benign.std(dim=0, keepdim=True, unbiased=False)
        byz = (mean_b - 1.5 * std_b).expand(w.f, cols)
    elif w.attack == "mix":
        h = w.f // 2
        byz = torch.cat([signflip(h), gaussian(w.f - h)], dim=0)
    else:
        raise ValueError(f"unknown attack {w.attack!r}")
    out[nb:] = byz
    return out


def num_tiles(w: Workload) -> int:
    return (w.d + TILE - 1) // TILE


def generate(w: Workload, device, ld: int | None = None) -> torch.Tensor:
    """The whole n x d matrix on `device`; row pitch `ld` elements (default d).

    Returns a view of shape (n, d) into an (n, ld) allocation.
    """
    ld = w.d if ld is None else int(ld)
    if ld < w.d:
        raise ValueError("ld must be >= d")
    store = torch.empty(w.n, max(ld, 1), device=device, dtype=torch.float32)
    if ld > w.d:
        store[:, w.d:] = float("nan")   # padding must never influence a result
    for t in range(num_tiles(w)):
        lo = t * TILE
        hi = min(w.d, lo + TILE)
        store[:, lo:hi] = generate_tile(w, t, device)
    return store[:, : w.d]


def checksum(x: torch.Tensor) -> int:
    """64-bit wrap-around sum of the input's 32-bit words (identifies the bytes in reports)."""
    total = 0
    flat = x if x.dim() == 2 else x.reshape(1, -1)
    for i in range(flat.shape[0]):
        total += int(flat[i].contiguous().view(torch.int32).sum(dtype=torch.int64).item())
    return total & ((1 << 64) - 1)
