"""CPU oracle for BRACE robust chunk aggregation -- TEST INFRASTRUCTURE ONLY.

This module is the slow, plain, obviously-correct statement of what the GPU
path must compute.  It is imported only by tests/, by the smoke check and by
the benchmark's cpu_baseline leg; the product path (the HIP library and its
Python binding) never imports, links or calls it, and it never imports them.

Everything is numpy on the host, integers in int64 and floating sums in
float64.  There is no blocking, fusion or reordering beyond what the paper's
definition states.

What follows the paper, and where:

* sign quantisation ............ Sec. 3, Phase I (Quantization)
* ring Share-Reduce ............ Sec. 2.2 Phase I; Sec. 3 Phase II
* consensus map ................ Sec. 3 Phase III, Eq. (1); restated in
                                 App. A as 2*I(sum > lambda) - 1
* ring Share-Only .............. Sec. 2.2 Phase II; Sec. 3 Phase IV
* chunk partition .............. Sec. 2.2 (n sub-vectors of about equal size)
* communication cost ........... Sec. 2.1 (SC), Sec. 2.2 (RAR), Sec. 3 / Table 1
* Mean rule, model update ...... Sec. 2.1; Sec. 2.2; App. A (update rule)
* ring-order float sum ......... Sec. 2.2 Share-Reduce (the receiver adds its own
                                 sub-vector), in the clients' own precision

Readings taken where the paper is silent (each is switchable or checked by a
test, none is pinned by a printed value):

* sign(+0) = sign(-0) = 0 and sign(NaN) = 0 by default; `zero_sign` in
  {-1, 0, +1} replaces that value.                       [parity unpinned]
* when n does not divide d the first (d mod n) chunks hold one more
  coordinate than the rest.                              [parity unpinned]
* packed output: bit j of byte b is coordinate 8*b + j, 1 means +1.
                                                         [parity unpinned]
* one-bit form (vote_plane): bit = 1 where the vote is +1, LSB first, rows padded
  to 16 bytes; same status as the two-plane layout below.   [parity unpinned]
* precision of the plain ring sum: the paper counts m bits per dimension and never
  names a floating format; reading: the clients hold fp32 (m = 32, as in the traffic
  example of Sec. 3) and add in it.  The ORDER of the additions is pinned by the
  three-client example; the format is this build's reading.
* bit planes of the quantise-once form (sign_planes): per client, word pair j
  = ("x > 0" bits, "x < 0" bits) of coordinates 32j .. 32j+31, LSB first, rows
  padded to an even number of pairs.  A storage convention of this build, not
  of the paper; what is computed from the planes is pinned through Eq. (1).
                                                         [parity unpinned]
Pinned by the paper: Eq. (1) itself incl. the tie sum == lambda -> -1, the
ring direction and chunk ownership (three-client example of Sec. 2.2), the
attacked sum [22, 1, -185] (Sec. 3), the traffic closed forms (Table 1) and
the fact that every client ends with the same vector (Sec. 3 Phase IV).
"""

from __future__ import annotations

from dataclasses import dataclass, field
from fractions import Fraction

import numpy as np


# --------------------------------------------------------------------------
# Chunk partition and ring ownership (Sec. 2.2; three-client example)
# --------------------------------------------------------------------------

def chunk_range(n: int, d: int, c: int) -> tuple[int, int]:
    """Half-open coordinate range [lo, hi) of ring chunk c (0-indexed).

    Sec. 2.2 only asks for n sub-vectors of about the same size.
    Reading: chunks are contiguous and ascending; with q = d div n and
    r = d mod n the first r chunks have q + 1 coordinates, the others q.
    """
    if n < 1 or d < 0 or not (0 <= c < n):
        raise ValueError("chunk_range: need n >= 1, d >= 0, 0 <= c < n")
    q, r = divmod(d, n)
    lo = c * q + min(c, r)
    hi = lo + q + (1 if c < r else 0)
    return lo, hi


def chunk_owner(n: int, c: int) -> int:
    """Client (0-indexed) that holds the fully reduced chunk c after Share-Reduce.

    In the three-client example of Sec. 2.2 Client 1 ends with the second
    sub-vector, i.e. 1-indexed chunk c sits on client c - 1; 0-indexed that is
    client (c - 1) mod n.
    """
    if n < 1 or not (0 <= c < n):
        raise ValueError("chunk_owner: need n >= 1, 0 <= c < n")
    return (c - 1) % n


# --------------------------------------------------------------------------
# Phase I and Phase III as stand-alone maps
# --------------------------------------------------------------------------

def sign_quantize(g: np.ndarray, zero_sign: int = 0) -> np.ndarray:
    """Element-wise sign of a gradient (Sec. 3, Phase I), as int64.

    x > 0 -> +1, x < 0 -> -1, everything else (+0, -0, NaN) -> zero_sign.
    Infinities and denormals keep their sign.
    """
    if zero_sign not in (-1, 0, 1):
        raise ValueError("zero_sign must be -1, 0 or +1")
    g = np.asarray(g)
    s = np.full(g.shape, zero_sign, dtype=np.int64)
    s[g > 0] = 1
    s[g < 0] = -1
    return s


def consensus(sums: np.ndarray, lam: float) -> np.ndarray:
    """Eq. (1): +1 where the sign-sum exceeds lambda, -1 otherwise (float32).

    The sums are small integers, so the comparison in float64 is exact.
    """
    lam = float(lam)
    if not np.isfinite(lam):
        raise ValueError("lambda must be finite")
    sums = np.asarray(sums, dtype=np.int64)
    return np.where(sums.astype(np.float64) > lam, 1.0, -1.0).astype(np.float32)


def pack_bits(out: np.ndarray) -> np.ndarray:
    """1-bit-per-dimension form of a +-1 vector: bit j of byte b <- coordinate 8b+j."""
    out = np.asarray(out)
    d = out.shape[0]
    nbytes = (d + 7) // 8
    packed = np.zeros(nbytes, dtype=np.uint8)
    for j in range(8):
        col = out[j::8] > 0
        packed[: col.shape[0]] |= (col.astype(np.uint8) << j).astype(np.uint8)
    return packed


# --------------------------------------------------------------------------
# Oracle A: the definition, coordinate by coordinate
# --------------------------------------------------------------------------

@dataclass
class BraceResult:
    out: np.ndarray    # float32, +-1, length d
    sums: np.ndarray   # int64 sign-sums S[k], length d
    bits: np.ndarray   # uint8, ceil(d/8) bytes


def brace_direct(updates: np.ndarray, lam: float, zero_sign: int = 0) -> BraceResult:
    """GAR(g_1..g_n)[k] by Eq. (1) for every k; updates has shape (n, d)."""
    updates = np.asarray(updates)
    if updates.ndim != 2 or updates.shape[0] < 1:
        raise ValueError("updates must be (n, d) with n >= 1")
    sums = sign_quantize(updates, zero_sign).sum(axis=0, dtype=np.int64)
    out = consensus(sums, lam)
    return BraceResult(out=out, sums=sums, bits=pack_bits(out))


def brace_direct_loops(updates, lam: float, zero_sign: int = 0) -> list[float]:
    """The same definition in pure Python loops (tiny inputs only).

    Kept separate from brace_direct so that the vectorised version has an
    independent statement to be checked against.
    """
    n = len(updates)
    d = len(updates[0]) if n else 0
    res = []
    for k in range(d):
        total = 0
        for i in range(n):
            x = float(updates[i][k])
            if x > 0:
                total += 1
            elif x < 0:
                total -= 1
            else:
                total += zero_sign
        res.append(1.0 if total > lam else -1.0)
    return res


def brace_chunk(updates: np.ndarray, c: int, lam: float, zero_sign: int = 0):
    """Aggregate of ring chunk c only: returns (lo, hi, out[lo:hi], sums[lo:hi])."""
    updates = np.asarray(updates)
    n, d = updates.shape
    lo, hi = chunk_range(n, d, c)
    part = brace_direct(updates[:, lo:hi], lam, zero_sign)
    return lo, hi, part.out, part.sums


# --------------------------------------------------------------------------
# Oracle B: literal ring simulation (Sec. 2.2 and Sec. 3, Phases I-IV)
# --------------------------------------------------------------------------

@dataclass
class RingMessage:
    phase: str          # "share_reduce" or "share_only"
    step: int           # 1 .. n-1
    src: int            # 0-indexed client
    dst: int
    chunk: int          # 0-indexed chunk
    payload: np.ndarray


@dataclass
class RingResult:
    buffers: list             # per-client final vector (length d each)
    bits_sent: list           # per-client total bits put on the wire
    owned_after_reduce: list  # per client: (chunk index, reduced chunk values)
    messages: list = field(default_factory=list)


def ring_all_reduce(updates: np.ndarray, mode: str = "brace", lam: float = 0.0,
                    zero_sign: int = 0, m_bits: int = 32,
                    record: bool = False, dtype=np.float64) -> RingResult:
    """Run the n-client ring exactly as the text describes it.

    mode "sum":   plain RAR (Sec. 2.2) -- floating addition, no quantisation.  `dtype` is the
                  precision the clients hold and add their sub-vectors in: float64 gives the
                  mathematical sum up to double rounding, float32 what a ring of clients with
                  m = 32-bit gradients delivers (Sec. 2.2 lets every receiver add the incoming
                  sub-vector to its own, so chunk c is accumulated in the order
                  c, c+1, ..., c-1 (mod n), one rounding per step).
    mode "brace": Phase I sign, Phase II integer addition of signs, Phase III
                  Eq. (1) on the owned chunk, Phase IV circulate the result.

    All clients act at once in each step: every message of a step is built
    from the state before that step, then delivered.  Client i's downstream
    neighbour is (i + 1) mod n.  In Share-Reduce step s client i forwards
    chunk (i - (s - 1)) mod n; in Share-Only step s it forwards chunk
    (i + 2 - s) mod n.  Wire cost: m_bits per dimension, except BRACE's
    Share-Only which carries 1 bit per dimension (Sec. 3, cost paragraph).
    """
    updates = np.asarray(updates)
    n, d = updates.shape
    if mode not in ("sum", "brace"):
        raise ValueError("mode must be 'sum' or 'brace'")
    ranges = [chunk_range(n, d, c) for c in range(n)]

    if mode == "brace":
        buf = [sign_quantize(updates[i], zero_sign) for i in range(n)]   # Phase I
    else:
        buf = [updates[i].astype(dtype) for i in range(n)]
    sent = [0] * n
    log = []

    # Share-Reduce: n-1 steps, receiver adds.
    for s in range(1, n):
        msgs = []
        for i in range(n):
            c = (i - (s - 1)) % n
            lo, hi = ranges[c]
            msgs.append((i, (i + 1) % n, c, buf[i][lo:hi].copy()))
        for src, dst, c, payload in msgs:
            lo, hi = ranges[c]
            buf[dst][lo:hi] = buf[dst][lo:hi] + payload
            sent[src] += (hi - lo) * m_bits
            if record:
                log.append(RingMessage("share_reduce", s, src, dst, c, payload))

    owned = []
    for i in range(n):
        c = (i + 1) % n
        lo, hi = ranges[c]
        owned.append((c, buf[i][lo:hi].copy()))

    # Consensus on the owned chunk (BRACE only).
    share_bits = m_bits
    if mode == "brace":
        share_bits = 1
        final = [np.zeros(d, dtype=np.float32) for _ in range(n)]
        for i in range(n):
            c = (i + 1) % n
            lo, hi = ranges[c]
            final[i][lo:hi] = consensus(buf[i][lo:hi], lam)
        buf = final

    # Share-Only: n-1 steps, receiver overwrites.
    for s in range(1, n):
        msgs = []
        for i in range(n):
            c = (i + 2 - s) % n
            lo, hi = ranges[c]
            msgs.append((i, (i + 1) % n, c, buf[i][lo:hi].copy()))
        for src, dst, c, payload in msgs:
            lo, hi = ranges[c]
            buf[dst][lo:hi] = payload
            sent[src] += (hi - lo) * share_bits
            if record:
                log.append(RingMessage("share_only", s, src, dst, c, payload))

    return RingResult(buffers=buf, bits_sent=sent, owned_after_reduce=owned,
                      messages=log)


# --------------------------------------------------------------------------
# Communication cost closed forms (Sec. 2.1, Sec. 2.2, Sec. 3, Table 1)
# --------------------------------------------------------------------------

def cost_sc(m: int, n: int, d: int) -> Fraction:
    return Fraction(m * n * d)


def cost_rar(m: int, n: int, d: int) -> Fraction:
    return Fraction(2 * m * d * (n - 1), n)


def cost_brace(m: int, n: int, d: int) -> Fraction:
    return Fraction(d * (n - 1) * (m + 1), n)


# --------------------------------------------------------------------------
# The operation BRACE replaces, and the consumer of its result
# --------------------------------------------------------------------------

def rar_sum_direct(updates: np.ndarray) -> np.ndarray:
    """sum_i g_i in float64 (what plain RAR delivers to every client, Sec. 2.2)."""
    return np.asarray(updates, dtype=np.float64).sum(axis=0)


def rar_sum_ring_order(updates: np.ndarray, dtype=np.float32) -> np.ndarray:
    """What plain RAR delivers when the clients add in `dtype` (Sec. 2.2, Share-Reduce).

    Chunk c starts as client c's own sub-vector; in step s the next client on the ring adds
    its own sub-vector to what it received.  So coordinate k of chunk c ends as
        (((g_c[k] + g_{c+1}[k]) + g_{c+2}[k]) + ...) + g_{c-1}[k]      (indices mod n),
    every + rounded to `dtype`.  This is the same arithmetic as ring_all_reduce(mode="sum",
    dtype=dtype), written per chunk instead of per message.
    """
    updates = np.asarray(updates)
    n, d = updates.shape
    out = np.zeros(d, dtype=dtype)
    for c in range(n):
        lo, hi = chunk_range(n, d, c)
        acc = updates[c, lo:hi].astype(dtype)
        for step in range(1, n):
            acc = (acc + updates[(c + step) % n, lo:hi].astype(dtype)).astype(dtype)
        out[lo:hi] = acc
    return out


def mean_ring_order(updates: np.ndarray, dtype=np.float32) -> np.ndarray:
    """The Mean rule of Sec. 2.1 on top of the ring-order sum: one division by n in `dtype`."""
    updates = np.asarray(updates)
    total = rar_sum_ring_order(updates, dtype)
    return (total / dtype(updates.shape[0])).astype(dtype)


def mean_direct(updates: np.ndarray) -> np.ndarray:
    """The Mean aggregation rule of Sec. 2.1 in float64."""
    updates = np.asarray(updates, dtype=np.float64)
    return updates.sum(axis=0) / updates.shape[0]


def model_update(w: np.ndarray, agg: np.ndarray, eta: float) -> np.ndarray:
    """w <- w - eta * GAR(...) in float64 (Sec. 2.1; App. A update rule)."""
    return np.asarray(w, dtype=np.float64) - float(eta) * np.asarray(agg, dtype=np.float64)


# --------------------------------------------------------------------------
# Quantise-once form: Phase I materialised as bit planes, Phases II-IV on the planes
# --------------------------------------------------------------------------

def packed_row_words(d: int) -> int:
    """32-bit words per client row of the packed sign matrix: an even number of
    (positive, negative) word pairs, so that rows stay 16-byte aligned."""
    w = (d + 31) // 32
    w += w & 1
    return 2 * w


def sign_planes(updates: np.ndarray) -> np.ndarray:
    """Sec. 3 Phase I kept as data: per client two bit planes, "x > 0" and "x < 0".

    Returns uint32 of shape (n, packed_row_words(d)); word pair j = (positive bits,
    negative bits) of coordinates 32j .. 32j+31, bit b <-> coordinate 32j + b.  A
    coordinate that is +-0 or NaN has neither bit set; padding bits are zero.
    """
    updates = np.asarray(updates)
    n, d = updates.shape
    words = packed_row_words(d)
    out = np.zeros((n, words), dtype=np.uint32)
    for plane, mask in ((0, updates > 0), (1, updates < 0)):
        padded = np.zeros((n, (words // 2) * 32), dtype=np.uint8)
        padded[:, :d] = mask
        packed = np.packbits(padded, axis=1, bitorder="little")        # bytes, LSB first
        out[:, plane::2] = packed.view("<u4").reshape(n, words // 2)
    return out


def brace_from_planes(planes: np.ndarray, d: int, lam: float, zero_sign: int = 0) -> BraceResult:
    """Phases II-IV from the bit planes: S = #pos - #neg + zero_sign * #neither, then Eq. (1)."""
    planes = np.asarray(planes, dtype=np.uint32)
    n = planes.shape[0]

    def unpack(plane):
        words = np.ascontiguousarray(planes[:, plane::2]).astype("<u4")
        bits = np.unpackbits(words.view(np.uint8).reshape(n, -1), axis=1, bitorder="little")
        return bits[:, :d].astype(np.int64)

    pos, neg = unpack(0), unpack(1)
    sums = (pos - neg + zero_sign * (1 - pos - neg)).sum(axis=0)
    out = consensus(sums, lam)
    return BraceResult(out=out, sums=sums, bits=pack_bits(out))


# --------------------------------------------------------------------------
# signSGD run over the same four phases (Sec. 5.2): plain majority vote
# --------------------------------------------------------------------------

def vote_plane_row_words(d: int) -> int:
    """32-bit words per client row of the one-bit form, padded to 16 bytes."""
    w = (d + 31) // 32
    return (w + 3) // 4 * 4


def vote_plane(updates: np.ndarray, zero_sign: int) -> np.ndarray:
    """Sec. 3 Phase I as the paper words it, one bit per dimension: bit = 1 where the client's
    quantised vote is +1.  Only defined when every coordinate votes, i.e. zero_sign = +1 or -1
    (with zero_sign = 0 a zero abstains and one bit cannot say so).

    Returns uint32 of shape (n, vote_plane_row_words(d)); bit b of word j <-> coordinate
    32j + b; padding bits are zero.
    """
    if zero_sign not in (-1, 1):
        raise ValueError("the one-bit form needs zero_sign = +1 or -1")
    updates = np.asarray(updates)
    n, d = updates.shape
    words = vote_plane_row_words(d)
    padded = np.zeros((n, words * 32), dtype=np.uint8)
    padded[:, :d] = sign_quantize(updates, zero_sign) > 0
    packed = np.packbits(padded, axis=1, bitorder="little")            # bytes, LSB first
    return packed.view("<u4").reshape(n, words).astype(np.uint32)


def brace_from_vote_plane(plane: np.ndarray, d: int, lam: float) -> BraceResult:
    """Phases II-IV from the one-bit votes: with P clients voting +1 out of n, the sign-sum is
    S = P - (n - P) = 2P - n, then Eq. (1)."""
    plane = np.asarray(plane, dtype=np.uint32)
    n = plane.shape[0]
    as_bytes = np.ascontiguousarray(plane).astype("<u4").view(np.uint8).reshape(n, -1)
    ups = np.unpackbits(as_bytes, axis=1, bitorder="little")[:, :d].astype(np.int64)
    sums = 2 * ups.sum(axis=0) - n
    out = consensus(sums, lam)
    return BraceResult(out=out, sums=sums, bits=pack_bits(out))


def signsgd_majority(updates: np.ndarray, zero_sign: int = 0) -> np.ndarray:
    """sign(sum_i sign(g_i[k])) in {-1, 0, +1} as float32: Phase III replaced by the plain
    sign, ties left at 0.  Where the sum is not zero this is Eq. (1) with lambda = 0."""
    sums = sign_quantize(np.asarray(updates), zero_sign).sum(axis=0, dtype=np.int64)
    return np.sign(sums).astype(np.float32)
