"""Thin ctypes binding of libbrace.so: argument marshalling only.

Every step of the aggregation runs inside the HIP library.  Tensors are used
for their device pointer, shape and pitch; PyTorch supplies device memory and
the stream, nothing else.  If the library has not been built this module
raises -- there is no fallback path.
"""

from __future__ import annotations

import ctypes
import os

PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG, "libbrace.so")

BRACE_OK, BRACE_EINVAL, BRACE_ERANGE, BRACE_EHIP = 0, 1, 2, 3
BRACE_MAX_CLIENTS = 32767


class BraceParams(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("lambda_", ctypes.c_float),
        ("zero_sign", ctypes.c_int32),
        ("rule", ctypes.c_int32),
        ("ld", ctypes.c_int64),
        ("out_bits_dev", ctypes.c_void_p),
        ("sums_dev", ctypes.c_void_p),
    ]


class BraceTuning(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("vec", ctypes.c_int32),
        ("cols", ctypes.c_int32),
        ("unroll", ctypes.c_int32),
        ("nontemporal", ctypes.c_int32),
        ("pipeline", ctypes.c_int32),
        ("split_writes", ctypes.c_int32),
        ("rowsplit", ctypes.c_int32),
        ("stage_writes", ctypes.c_int32),
    ]


class BraceRarParams(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("mean", ctypes.c_int32),
        ("ld", ctypes.c_int64),
        ("order", ctypes.c_int32),
        ("reserved", ctypes.c_int32),
    ]


class BraceError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"brace status {code}: {text}")
        self.code = code
        self.text = text


_lib = None

EXPORTS = (
    "brace_params_init", "brace_aggregate", "brace_aggregate_chunk", "brace_chunk_range",
    "brace_chunk_owner", "brace_last_error", "brace_set_tuning", "brace_get_tuning",
    "brace_probe_read", "brace_probe_copy", "brace_rar_aggregate", "brace_rar_aggregate_chunk",
    "brace_aggregate_update", "brace_aggregate_update_chunk", "brace_expand_bits", "brace_apply_bits",
    "brace_packed_row_words", "brace_quantize", "brace_vote_packed", "brace_vote_packed_chunk",
    "brace_vote_packed_chunks", "brace_aggregate_chunks", "brace_consensus_sums",
    "brace_set_pointer_checks", "brace_init_device", "brace_comm_cost",
    "brace_1bit_row_words", "brace_quantize_1bit", "brace_vote_1bit", "brace_vote_1bit_chunks",
    "brace_packed_row_pitch", "brace_1bit_row_pitch", "brace_rar_params_init", "brace_threshold",
    "brace_aggregate_update_noalloc",
)


def lib():
    """The loaded shared library (raises if it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2501_17392_amd.build` "
            "(there is no non-HIP fallback)")
    # One process must hold ONE HIP runtime.  PyTorch ships its own libamdhip64 (same
    # soname as the system one); importing torch first makes the dynamic loader bind
    # libbrace.so to that already-loaded runtime, so device pointers and streams handed
    # over from torch are valid in the library.  Loaded the other way round, the process
    # ends up with two runtimes and the second one sees no device.
    import torch  # noqa: F401
    L = ctypes.CDLL(LIB_PATH)
    i64, vp = ctypes.c_int64, ctypes.c_void_p
    pp = ctypes.POINTER(BraceParams)
    L.brace_params_init.argtypes = [pp]
    L.brace_params_init.restype = None
    L.brace_aggregate.argtypes = [vp, i64, i64, i64, pp, vp, vp]
    L.brace_aggregate.restype = ctypes.c_int
    L.brace_aggregate_chunk.argtypes = [vp, i64, i64, i64, i64, pp, vp, vp]
    L.brace_aggregate_chunk.restype = ctypes.c_int
    L.brace_aggregate_chunks.argtypes = [vp, i64, i64, i64, i64, i64, pp, vp, vp]
    L.brace_aggregate_chunks.restype = ctypes.c_int
    L.brace_chunk_range.argtypes = [i64, i64, i64, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    L.brace_chunk_range.restype = ctypes.c_int
    L.brace_chunk_owner.argtypes = [i64, i64, ctypes.POINTER(i64)]
    L.brace_chunk_owner.restype = ctypes.c_int
    L.brace_last_error.argtypes = []
    L.brace_last_error.restype = ctypes.c_char_p
    L.brace_set_tuning.argtypes = [ctypes.POINTER(BraceTuning)]
    L.brace_set_tuning.restype = ctypes.c_int
    L.brace_get_tuning.argtypes = [ctypes.POINTER(BraceTuning)]
    L.brace_get_tuning.restype = ctypes.c_int
    L.brace_probe_read.argtypes = [vp, i64, ctypes.c_int32, vp, vp]
    L.brace_probe_read.restype = ctypes.c_int
    L.brace_probe_copy.argtypes = [vp, vp, i64, vp]
    L.brace_probe_copy.restype = ctypes.c_int
    L.brace_aggregate_update.argtypes = [vp, i64, i64, i64, pp, ctypes.c_float, vp, vp]
    L.brace_aggregate_update.restype = ctypes.c_int
    L.brace_aggregate_update_chunk.argtypes = [vp, i64, i64, i64, i64, pp, ctypes.c_float, vp, vp]
    L.brace_aggregate_update_chunk.restype = ctypes.c_int
    L.brace_aggregate_update_noalloc.argtypes = [vp, i64, i64, i64, pp, ctypes.c_float, vp, vp]
    L.brace_aggregate_update_noalloc.restype = ctypes.c_int
    L.brace_expand_bits.argtypes = [vp, i64, vp, vp]
    L.brace_expand_bits.restype = ctypes.c_int
    L.brace_apply_bits.argtypes = [vp, i64, ctypes.c_float, vp, vp]
    L.brace_apply_bits.restype = ctypes.c_int
    L.brace_packed_row_words.argtypes = [i64]
    L.brace_packed_row_words.restype = ctypes.c_int64
    L.brace_quantize.argtypes = [vp, i64, i64, i64, vp, i64, vp]
    L.brace_quantize.restype = ctypes.c_int
    L.brace_vote_packed.argtypes = [vp, i64, i64, i64, i64, pp, vp, vp]
    L.brace_vote_packed.restype = ctypes.c_int
    L.brace_vote_packed_chunk.argtypes = [vp, i64, i64, i64, i64, i64, pp, vp, vp]
    L.brace_vote_packed_chunk.restype = ctypes.c_int
    L.brace_vote_packed_chunks.argtypes = [vp, i64, i64, i64, i64, i64, i64, pp, vp, vp]
    L.brace_vote_packed_chunks.restype = ctypes.c_int
    L.brace_consensus_sums.argtypes = [vp, i64, i64, i64, pp, vp, vp]
    L.brace_consensus_sums.restype = ctypes.c_int
    L.brace_set_pointer_checks.argtypes = [ctypes.c_int32]
    L.brace_set_pointer_checks.restype = ctypes.c_int
    L.brace_init_device.argtypes = []
    L.brace_init_device.restype = ctypes.c_int
    L.brace_comm_cost.argtypes = [ctypes.c_int32, i64, i64, i64, ctypes.POINTER(ctypes.c_double)]
    L.brace_comm_cost.restype = ctypes.c_int
    L.brace_1bit_row_words.argtypes = [i64]
    L.brace_1bit_row_words.restype = i64
    L.brace_quantize_1bit.argtypes = [vp, i64, i64, i64, ctypes.c_int32, vp, i64, vp]
    L.brace_quantize_1bit.restype = ctypes.c_int
    L.brace_vote_1bit.argtypes = [vp, i64, i64, i64, i64, pp, vp, vp]
    L.brace_vote_1bit.restype = ctypes.c_int
    L.brace_vote_1bit_chunks.argtypes = [vp, i64, i64, i64, i64, i64, i64, pp, vp, vp]
    L.brace_vote_1bit_chunks.restype = ctypes.c_int
    L.brace_packed_row_pitch.argtypes = [i64]
    L.brace_packed_row_pitch.restype = i64
    L.brace_1bit_row_pitch.argtypes = [i64]
    L.brace_1bit_row_pitch.restype = i64
    L.brace_threshold.argtypes = [i64, ctypes.c_float, ctypes.POINTER(ctypes.c_int32)]
    L.brace_threshold.restype = ctypes.c_int
    rp = ctypes.POINTER(BraceRarParams)
    L.brace_rar_params_init.argtypes = [rp]
    L.brace_rar_params_init.restype = None
    L.brace_rar_aggregate.argtypes = [vp, i64, i64, rp, vp, vp]
    L.brace_rar_aggregate.restype = ctypes.c_int
    L.brace_rar_aggregate_chunk.argtypes = [vp, i64, i64, i64, rp, vp, vp]
    L.brace_rar_aggregate_chunk.restype = ctypes.c_int
    _lib = L
    return L


def brace_last_error() -> str:
    return lib().brace_last_error().decode()


def _check(rc: int):
    if rc != BRACE_OK:
        raise BraceError(rc, brace_last_error())


def make_params(lam: float = 5.0, zero_sign: int = 0, ld: int = 0,
                out_bits_ptr: int | None = None, sums_ptr: int | None = None,
                rule: int = 0) -> BraceParams:
    p = BraceParams()
    lib().brace_params_init(ctypes.byref(p))
    p.lambda_ = float(lam)
    p.zero_sign = int(zero_sign)
    p.rule = int(rule)
    p.ld = int(ld)
    p.out_bits_dev = out_bits_ptr
    p.sums_dev = sums_ptr
    return p


def brace_chunk_range(n: int, d: int, chunk: int) -> tuple[int, int]:
    lo, hi = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().brace_chunk_range(n, d, chunk, ctypes.byref(lo), ctypes.byref(hi)))
    return lo.value, hi.value


def brace_threshold(n: int, lam: float) -> int:
    """Integer threshold T of Eq. (1): S > lam <=> S >= T for sign-sums over n clients."""
    t = ctypes.c_int32()
    _check(lib().brace_threshold(n, float(lam), ctypes.byref(t)))
    return t.value


def brace_chunk_owner(n: int, chunk: int) -> int:
    o = ctypes.c_int64()
    _check(lib().brace_chunk_owner(n, chunk, ctypes.byref(o)))
    return o.value


def _stream_handle(stream) -> int | None:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if hasattr(stream, "cuda_stream"):
        return stream.cuda_stream
    return int(stream)


def _ptr(t) -> int | None:
    return None if t is None else t.data_ptr()


def _dev(t, name: str, dtypes):
    """Device pointer of an optional flat buffer after checking what the C side cannot see:
    that it is a CUDA tensor of the element type the ABI reads or writes, and contiguous.
    (Sizes are checked by the library against the allocation that holds the pointer.)"""
    if t is None:
        return None
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise ValueError(f"{name} must be a CUDA tensor")
    if t.dtype not in dtypes:
        raise ValueError(f"{name} must have dtype {' or '.join(str(x) for x in dtypes)}, "
                         f"not {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _f32(t, name, d=0):
    import torch
    return _dev(t, name, (torch.float32,))


def _i16(t, name, d=0):
    import torch
    return _dev(t, name, (torch.int16,))


def _bitbuf(t, name, d=0):
    """Packed result: any integer storage of 4*ceil(d/32) bytes."""
    import torch
    return _dev(t, name, (torch.int32, torch.uint8, torch.int8, torch.int16, torch.int64))


def _rows(t, name: str, dtype):
    """(rows, cols, pitch) of a row-major 2-D CUDA tensor with unit column stride."""
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != dtype:
        raise ValueError(f"{name} must be a CUDA tensor of dtype {dtype}")
    if t.dim() != 2 or (t.stride(1) != 1 and t.shape[1] > 1):
        raise ValueError(f"{name} must be 2-D with unit column stride")
    rows, cols = t.shape
    if rows > 1 and t.stride(0) < cols:
        raise ValueError(f"{name}: rows overlap (pitch {t.stride(0)} < {cols} columns)")
    return rows, cols, (t.stride(0) if rows > 1 else max(cols, 1))


def _matrix(updates):
    import torch
    return _rows(updates, "updates", torch.float32)


def _planes(t, name: str):
    """(n, pitch in words) of a packed matrix; a single row is passed as dense."""
    import torch
    n, _, pitch = _rows(t, name, torch.int32)
    return n, (pitch if n > 1 else 0)


def brace_aggregate(updates, f: int, lam: float = 5.0, zero_sign: int = 0, out=None,
                    out_bits=None, sums=None, stream=None, rule: int = 0):
    """brace_aggregate of the C ABI on device tensors; returns `out`.

    updates: (n, d) float32 device tensor, unit column stride, any row pitch >= d.
    out: float32[d], out_bits: int32/uint8 storage of 4*ceil(d/32) bytes, sums: int16[d].
    """
    n, d, ld = _matrix(updates)
    p = make_params(lam, zero_sign, ld, _bitbuf(out_bits, "out_bits", d), _i16(sums, "sums", d), rule)
    _check(lib().brace_aggregate(updates.data_ptr(), n, d, f, ctypes.byref(p), _f32(out, "out", d),
                                 _stream_handle(stream)))
    return out


def brace_aggregate_chunk(updates, f: int, chunk: int, lam: float = 5.0, zero_sign: int = 0,
                          out=None, out_bits=None, sums=None, stream=None, rule: int = 0):
    """brace_aggregate_chunk of the C ABI; `out` etc. are the FULL length-d vectors."""
    n, d, ld = _matrix(updates)
    p = make_params(lam, zero_sign, ld, _bitbuf(out_bits, "out_bits", d), _i16(sums, "sums", d), rule)
    _check(lib().brace_aggregate_chunk(updates.data_ptr(), n, d, f, chunk, ctypes.byref(p),
                                       _f32(out, "out", d), _stream_handle(stream)))
    return out


def brace_set_tuning(vec: int = 0, cols: int = 0, unroll: int = 0, nontemporal: int = 1,
                     pipeline: int = 1, split_writes: int = 0, rowsplit: int = 0,
                     stage_writes: int = 0):
    t = BraceTuning(ctypes.sizeof(BraceTuning), vec, cols, unroll, nontemporal, pipeline,
                    split_writes, rowsplit, stage_writes)
    _check(lib().brace_set_tuning(ctypes.byref(t)))


def brace_reset_tuning():
    _check(lib().brace_set_tuning(None))


def brace_get_tuning() -> dict:
    t = BraceTuning()
    _check(lib().brace_get_tuning(ctypes.byref(t)))
    return {k: getattr(t, k) for k, _ in BraceTuning._fields_ if k != "struct_size"}


def brace_probe_read(src, sink, nontemporal: int = 1, stream=None):
    """Streaming read of a whole device tensor (measurement aid)."""
    nbytes = src.numel() * src.element_size()
    _check(lib().brace_probe_read(src.data_ptr(), nbytes, int(nontemporal), sink.data_ptr(),
                                  _stream_handle(stream)))


def brace_probe_copy(dst, src, stream=None):
    """Plain copy of a whole device tensor (measurement aid)."""
    nbytes = src.numel() * src.element_size()
    _check(lib().brace_probe_copy(dst.data_ptr(), src.data_ptr(), nbytes, _stream_handle(stream)))


def brace_rar_aggregate(updates, out, mean: bool = False, chunk: int | None = None, stream=None,
                        order: int = 0):
    """Plain ring-all-reduce sum (or mean) of the n client rows; `out` is the full vector.
    order 0: fp64 accumulation in index order; order 1: fp32 in the ring order of each chunk."""
    n, d, ld = _matrix(updates)
    p = BraceRarParams()
    lib().brace_rar_params_init(ctypes.byref(p))
    p.mean, p.ld, p.order = (1 if mean else 0), ld, int(order)
    if chunk is None:
        _check(lib().brace_rar_aggregate(updates.data_ptr(), n, d, ctypes.byref(p),
                                         _f32(out, "out", d), _stream_handle(stream)))
    else:
        _check(lib().brace_rar_aggregate_chunk(updates.data_ptr(), n, d, chunk, ctypes.byref(p),
                                               _f32(out, "out", d), _stream_handle(stream)))
    return out


def brace_aggregate_update(updates, f: int, w, eta: float, lam: float = 5.0, zero_sign: int = 0,
                           out_bits=None, sums=None, chunk: int | None = None, stream=None,
                           rule: int = 0):
    """Vote fused with the model update w <- w - eta * result (in place); returns w."""
    n, d, ld = _matrix(updates)
    p = make_params(lam, zero_sign, ld, _bitbuf(out_bits, "out_bits", d), _i16(sums, "sums", d), rule)
    if chunk is None:
        _check(lib().brace_aggregate_update(updates.data_ptr(), n, d, f, ctypes.byref(p),
                                            float(eta), _f32(w, "w", d), _stream_handle(stream)))
    else:
        _check(lib().brace_aggregate_update_chunk(updates.data_ptr(), n, d, f, chunk,
                                                  ctypes.byref(p), float(eta), _f32(w, "w", d),
                                                  _stream_handle(stream)))
    return w


BRACE_NOALLOC_MAX_D = 1 << 27


def brace_aggregate_update_noalloc(updates, f: int, w, eta: float, lam: float = 5.0,
                                   zero_sign: int = 0, sums=None, stream=None, rule: int = 0):
    """brace_aggregate_update without a bit array: the bit-words live in the library's own
    per-device workspace (d <= BRACE_NOALLOC_MAX_D; calls on one device must not overlap)."""
    n, d, ld = _matrix(updates)
    p = make_params(lam, zero_sign, ld, None, _i16(sums, "sums", d), rule)
    _check(lib().brace_aggregate_update_noalloc(updates.data_ptr(), n, d, f, ctypes.byref(p),
                                                float(eta), _f32(w, "w", d), _stream_handle(stream)))
    return w


def brace_expand_bits(bits, d: int, out, stream=None):
    """Packed result -> d floats of +-1.0f."""
    _check(lib().brace_expand_bits(_bitbuf(bits, "bits", d), d, _f32(out, "out", d),
                                   _stream_handle(stream)))
    return out


def brace_apply_bits(bits, d: int, eta: float, w, stream=None):
    """Packed result applied to a model copy: w <- w - eta * (+-1)."""
    _check(lib().brace_apply_bits(_bitbuf(bits, "bits", d), d, float(eta), _f32(w, "w", d),
                                  _stream_handle(stream)))
    return w


def brace_packed_row_words(d: int) -> int:
    return int(lib().brace_packed_row_words(d))


def brace_packed_row_pitch(d: int) -> int:
    """Recommended row pitch (words) of the two-plane matrix: rows start on 128-byte lines."""
    return int(lib().brace_packed_row_pitch(d))


def brace_quantize(updates, signs, stream=None):
    """Phase I kept as data: (n, d) floats -> (n, brace_packed_row_words(d)) int32 bit planes."""
    n, d, ld = _matrix(updates)
    rows, ld_words = _planes(signs, "signs")
    if rows != n:
        raise ValueError("signs must have one row per client")
    _check(lib().brace_quantize(updates.data_ptr(), n, d, ld, signs.data_ptr(), ld_words,
                                _stream_handle(stream)))
    return signs


def brace_vote_packed(signs, d: int, f: int, lam: float = 5.0, zero_sign: int = 0, out=None,
                      out_bits=None, stream=None):
    """Phases II-IV on the packed sign planes; same result as brace_aggregate on the floats."""
    n, ld_words = _planes(signs, "signs")
    p = make_params(lam, zero_sign, 0, _bitbuf(out_bits, "out_bits", d), None)
    _check(lib().brace_vote_packed(signs.data_ptr(), n, d, ld_words, f, ctypes.byref(p),
                                   _f32(out, "out", d), _stream_handle(stream)))
    return out


def brace_vote_packed_chunk(signs, d: int, f: int, chunk: int, lam: float = 5.0, zero_sign: int = 0,
                            out=None, out_bits=None, stream=None):
    """brace_vote_packed for one ring chunk; `out` / `out_bits` are the FULL vectors."""
    n, ld_words = _planes(signs, "signs")
    p = make_params(lam, zero_sign, 0, _bitbuf(out_bits, "out_bits", d), None)
    _check(lib().brace_vote_packed_chunk(signs.data_ptr(), n, d, ld_words, f, chunk, ctypes.byref(p),
                                         _f32(out, "out", d), _stream_handle(stream)))
    return out


def brace_vote_packed_chunks(signs, d: int, f: int, chunk_begin: int, chunk_end: int,
                             lam: float = 5.0, zero_sign: int = 0, out=None, out_bits=None,
                             stream=None):
    """brace_vote_packed for a run of consecutive ring chunks in one call."""
    n, ld_words = _planes(signs, "signs")
    p = make_params(lam, zero_sign, 0, _bitbuf(out_bits, "out_bits", d), None)
    _check(lib().brace_vote_packed_chunks(signs.data_ptr(), n, d, ld_words, f, chunk_begin, chunk_end,
                                          ctypes.byref(p), _f32(out, "out", d),
                                          _stream_handle(stream)))
    return out


def brace_1bit_row_words(d: int) -> int:
    return int(lib().brace_1bit_row_words(d))


def brace_1bit_row_pitch(d: int) -> int:
    """Recommended row pitch (words) of the one-bit matrix: rows start on 128-byte lines."""
    return int(lib().brace_1bit_row_pitch(d))


def brace_quantize_1bit(updates, zero_sign: int, votes, stream=None):
    """Phase I as one bit per dimension (zero_sign = +1 or -1): bit = 1 where the vote is +1."""
    n, d, ld = _matrix(updates)
    rows, ld_words = _planes(votes, "votes")
    if rows != n:
        raise ValueError("votes must have one row per client")
    _check(lib().brace_quantize_1bit(updates.data_ptr(), n, d, ld, int(zero_sign), votes.data_ptr(),
                                     ld_words, _stream_handle(stream)))
    return votes


def brace_vote_1bit(votes, d: int, f: int, lam: float = 5.0, out=None, out_bits=None, stream=None):
    """Phases II-IV on the one-bit votes; equals brace_aggregate with the zero_sign they were made with."""
    n, ld_words = _planes(votes, "votes")
    p = make_params(lam, 0, 0, _bitbuf(out_bits, "out_bits", d), None)
    _check(lib().brace_vote_1bit(votes.data_ptr(), n, d, ld_words, f, ctypes.byref(p),
                                 _f32(out, "out", d), _stream_handle(stream)))
    return out


def brace_vote_1bit_chunks(votes, d: int, f: int, chunk_begin: int, chunk_end: int, lam: float = 5.0,
                           out=None, out_bits=None, stream=None):
    """brace_vote_1bit for a run of consecutive ring chunks; `out` / `out_bits` are the FULL vectors."""
    n, ld_words = _planes(votes, "votes")
    p = make_params(lam, 0, 0, _bitbuf(out_bits, "out_bits", d), None)
    _check(lib().brace_vote_1bit_chunks(votes.data_ptr(), n, d, ld_words, f, chunk_begin, chunk_end,
                                        ctypes.byref(p), _f32(out, "out", d),
                                        _stream_handle(stream)))
    return out


def brace_consensus_sums(parts, lam: float = 5.0, out=None, out_bits=None, stream=None):
    """Phase III on (g, d) int16 partial sign-sums: Eq. (1) applied to their column sums."""
    import torch
    g, d, ld = _rows(parts, "parts", torch.int16)
    p = make_params(lam, 0, 0, _bitbuf(out_bits, "out_bits", d), None)
    _check(lib().brace_consensus_sums(parts.data_ptr(), g, d, ld if g > 1 else 0, ctypes.byref(p),
                                      _f32(out, "out", d), _stream_handle(stream)))
    return out


def brace_aggregate_chunks(updates, f: int, chunk_begin: int, chunk_end: int, lam: float = 5.0,
                           zero_sign: int = 0, out=None, out_bits=None, sums=None, stream=None):
    """A run of consecutive ring chunks in one launch; `out` etc. are the FULL vectors."""
    n, d, ld = _matrix(updates)
    p = make_params(lam, zero_sign, ld, _bitbuf(out_bits, "out_bits", d), _i16(sums, "sums", d))
    _check(lib().brace_aggregate_chunks(updates.data_ptr(), n, d, f, chunk_begin, chunk_end,
                                        ctypes.byref(p), _f32(out, "out", d),
                                        _stream_handle(stream)))
    return out


BRACE_COST_SERVER_CLIENT, BRACE_COST_RING_ALL_REDUCE, BRACE_COST_BRACE = 0, 1, 2


def brace_comm_cost(scheme: int, m: int, n: int, d: int) -> float:
    """Bits per round of Table 1 for the given scheme (host arithmetic)."""
    v = ctypes.c_double()
    _check(lib().brace_comm_cost(scheme, m, n, d, ctypes.byref(v)))
    return v.value


def brace_init_device():
    """Host-side set-up for the current device (call once before capturing calls in a HIP graph)."""
    _check(lib().brace_init_device())


def brace_set_pointer_checks(enabled: bool):
    """Host-side validation of every device buffer before a launch (on by default)."""
    _check(lib().brace_set_pointer_checks(1 if enabled else 0))
