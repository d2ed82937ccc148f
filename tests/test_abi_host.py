"""The C ABI without a GPU: the library loads, exports what the header declares, and the
host-side arithmetic and argument validation behave as documented.  No kernel is launched:
every call here either is pure host arithmetic or is rejected before any HIP call."""

import ctypes
import os
import re

import pytest

from oracle import brace_oracle as O
from paper_2501_17392_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

FAKE_IN = 0x7F00_0000_0000     # never dereferenced: validation fails first
FAKE_OUT = 0x7F80_0000_0000


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(B.LIB_PATH):
        from paper_2501_17392_amd.build import build_library
        build_library()
    return B.lib()


def _declared_functions():
    names = []
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if fn.endswith(".h"):
            text = open(os.path.join(inc, fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names += re.findall(r"\b([a-z][a-z0-9_]*)\s*\([^;{]*\)\s*;", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol(L):
    declared = _declared_functions()
    assert "brace_aggregate" in declared and "brace_aggregate_chunk" in declared
    for name in declared:
        assert hasattr(L, name), f"{name} declared in include/ but not exported"
    assert set(B.EXPORTS) <= set(declared)


def test_method_header_holds_no_process_wide_state_calls():
    # include/brace.h is the method; tuning, the pointer-check switch and the probes are
    # process-wide state and measurement aids and live in include/brace_tuning.h.
    inc = os.path.join(ROOT, "include")
    method = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, "brace.h")).read(), flags=re.S)
    tuning = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, "brace_tuning.h")).read(), flags=re.S)
    for name in ("brace_set_tuning", "brace_get_tuning", "brace_probe_read", "brace_probe_copy",
                 "brace_set_pointer_checks", "brace_tuning_t"):
        assert name not in method, name
        assert name in tuning, name
    for name in ("brace_aggregate", "brace_aggregate_chunk", "brace_chunk_range", "brace_threshold",
                 "brace_rar_aggregate", "brace_aggregate_update_noalloc"):
        assert re.search(r"\b%s\s*\(" % name, method), name


def test_header_is_plain_c_and_host_entry_points_work_from_c(L, tmp_path):
    # gcc -std=c99 -pedantic on the header, a C program linked against the library, no GPU call.
    import subprocess
    exe = str(tmp_path / "abi_host")
    src = os.path.join(ROOT, "tests", "c", "abi_host.c")
    libdir = os.path.dirname(B.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic",
                    "-I", os.path.join(ROOT, "include"), src, "-o", exe,
                    "-L", libdir, "-lbrace", "-lm", f"-Wl,-rpath,{libdir}",
                    "-Wl,-rpath,/opt/rocm/lib"], check=True)
    res = subprocess.run([exe], capture_output=True, text=True)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "abi_host ok" in res.stdout


def test_host_planning_survives_random_arguments(L, tmp_path):
    """200,000 random calls (sizes up to 2^63, every alignment, every tuning) with the pointer
    checks off: on a machine without a GPU each call runs all of its host arithmetic and fails
    at the launch, so the program must end with status codes only.  (The same program linked
    against a host-sanitised build of the library is the overflow check; see tests/c/abi_fuzz.c.)"""
    import subprocess
    import torch
    if torch.cuda.device_count() > 0:
        pytest.skip("needs a machine without a GPU: the buffers are made-up addresses")
    exe = str(tmp_path / "abi_fuzz")
    src = os.path.join(ROOT, "tests", "c", "abi_fuzz.c")
    libdir = os.path.dirname(B.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-Werror",
                    "-I", os.path.join(ROOT, "include"), src, "-o", exe,
                    "-L", libdir, "-lbrace", "-lm", f"-Wl,-rpath,{libdir}",
                    "-Wl,-rpath,/opt/rocm/lib"], check=True)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "abi_fuzz ok" in res.stdout


def test_struct_layouts_match_the_header():
    assert ctypes.sizeof(B.BraceParams) == 40
    assert B.BraceParams.ld.offset == 16
    assert B.BraceParams.out_bits_dev.offset == 24
    assert B.BraceParams.sums_dev.offset == 32
    assert ctypes.sizeof(B.BraceTuning) == 36


def test_params_init_defaults(L):
    p = B.make_params()
    assert p.struct_size == ctypes.sizeof(B.BraceParams)
    assert p.lambda_ == 5.0 and p.zero_sign == 0 and p.ld == 0
    assert p.out_bits_dev is None and p.sums_dev is None


@pytest.mark.parametrize("n,d", [(1, 0), (1, 7), (3, 3), (10, 10_000), (20, 1_000_003),
                                 (50, 11_173_962), (100, 25_000_000), (64, 100_000_000), (7, 3)])
def test_chunk_range_and_owner_match_the_oracle(L, n, d):
    for c in sorted({0, 1 % n, n // 2, n - 1}):
        assert B.brace_chunk_range(n, d, c) == O.chunk_range(n, d, c)
        assert B.brace_chunk_owner(n, c) == O.chunk_owner(n, c)


def test_chunk_helpers_reject_bad_arguments(L):
    lo, hi = ctypes.c_int64(), ctypes.c_int64()
    assert L.brace_chunk_range(0, 5, 0, ctypes.byref(lo), ctypes.byref(hi)) == B.BRACE_EINVAL
    assert L.brace_chunk_range(3, -1, 0, ctypes.byref(lo), ctypes.byref(hi)) == B.BRACE_EINVAL
    assert L.brace_chunk_range(3, 5, 3, ctypes.byref(lo), ctypes.byref(hi)) == B.BRACE_ERANGE
    assert L.brace_chunk_range(3, 5, -1, ctypes.byref(lo), ctypes.byref(hi)) == B.BRACE_ERANGE
    assert L.brace_chunk_range(3, 5, 0, None, ctypes.byref(hi)) == B.BRACE_EINVAL
    assert "chunk" in B.brace_last_error() or "NULL" in B.brace_last_error()
    o = ctypes.c_int64()
    assert L.brace_chunk_owner(3, 3, ctypes.byref(o)) == B.BRACE_ERANGE
    assert L.brace_chunk_owner(0, 0, ctypes.byref(o)) == B.BRACE_EINVAL
    assert L.brace_chunk_owner(3, 0, None) == B.BRACE_EINVAL
    with pytest.raises(B.BraceError) as ei:
        B.brace_chunk_range(3, 5, 9)
    assert ei.value.code == B.BRACE_ERANGE


def _agg(L, *, inp=FAKE_IN, n=4, d=100, f=1, p="default", out=FAKE_OUT, chunk=None, **kw):
    if p == "default":
        p = B.make_params(**kw)
    pref = ctypes.byref(p) if p is not None else None
    if chunk is None:
        return L.brace_aggregate(inp, n, d, f, pref, out, None)
    return L.brace_aggregate_chunk(inp, n, d, f, chunk, pref, out, None)


def test_aggregate_rejects_invalid_arguments_before_touching_the_gpu(L):
    E, R = B.BRACE_EINVAL, B.BRACE_ERANGE
    assert _agg(L, p=None) == E
    assert _agg(L, inp=None) == E
    assert _agg(L, out=None) == E                       # no output at all
    assert _agg(L, n=0) == E
    assert _agg(L, n=-3) == E
    assert _agg(L, n=B.BRACE_MAX_CLIENTS + 1, f=0) == R
    assert _agg(L, d=-1) == E
    assert _agg(L, f=-1) == E
    assert _agg(L, f=5) == E                            # f > n
    assert _agg(L, lam=float("nan")) == E
    assert _agg(L, lam=float("inf")) == E
    assert _agg(L, zero_sign=2) == E
    assert _agg(L, zero_sign=-2) == E
    assert _agg(L, ld=99) == E                          # pitch smaller than d
    assert _agg(L, inp=FAKE_IN + 2) == E                # misaligned
    assert _agg(L, out=FAKE_OUT + 1) == E
    assert _agg(L, out_bits_ptr=FAKE_OUT + 0x1002) == E
    assert _agg(L, sums_ptr=FAKE_OUT + 0x2001) == E
    assert _agg(L, out=FAKE_IN + 4 * 150) == E          # out inside the input matrix
    bad = B.make_params()
    bad.struct_size = 12
    assert _agg(L, p=bad) == E
    assert "struct_size" in B.brace_last_error()
    assert _agg(L, rule=2) == E
    assert _agg(L, rule=-1) == E
    assert _agg(L, rule=1, out_bits_ptr=FAKE_OUT + 0x1000) == E   # no 1-bit form of {-1, 0, +1}
    assert _agg(L, chunk=4) == R
    assert _agg(L, chunk=-1) == R
    assert "chunk" in B.brace_last_error()


def test_chunk_run_validation(L):
    p = B.make_params()
    pr = ctypes.byref(p)
    R = B.BRACE_ERANGE
    assert L.brace_aggregate_chunks(FAKE_IN, 4, 100, 1, -1, 2, pr, FAKE_OUT, None) == R
    assert L.brace_aggregate_chunks(FAKE_IN, 4, 100, 1, 0, 5, pr, FAKE_OUT, None) == R
    assert L.brace_aggregate_chunks(FAKE_IN, 4, 100, 1, 3, 2, pr, FAKE_OUT, None) == R
    assert L.brace_aggregate_chunks(FAKE_IN, 4, 100, 1, 2, 2, pr, FAKE_OUT, None) == B.BRACE_OK
    assert L.brace_aggregate_chunks(FAKE_IN, 7, 3, 0, 4, 7, pr, FAKE_OUT, None) == B.BRACE_OK  # empty chunks
    assert L.brace_aggregate_chunks(None, 4, 100, 1, 0, 2, pr, FAKE_OUT, None) == B.BRACE_EINVAL


def test_degenerate_sizes_are_accepted_without_a_launch(L):
    assert _agg(L, d=0) == B.BRACE_OK                   # nothing to do
    assert _agg(L, d=0, inp=None, out=None) == B.BRACE_OK  # empty buffers may be NULL
    assert _agg(L, d=0, lam=float("nan")) == B.BRACE_EINVAL  # scalars are still checked
    assert _agg(L, n=7, d=3, f=0, chunk=5) == B.BRACE_OK  # d < n: chunk 5 is empty
    assert _agg(L, n=4, d=0, f=4) == B.BRACE_OK         # f = n is allowed; the rule ignores f


def test_update_and_bits_entry_points_validate(L):
    E, R = B.BRACE_EINVAL, B.BRACE_ERANGE
    p = B.make_params()
    pr = ctypes.byref(p)
    nan = ctypes.c_float(float("nan"))
    eta = ctypes.c_float(0.1)
    assert L.brace_aggregate_update(FAKE_IN, 4, 100, 1, pr, nan, FAKE_OUT, None) == E
    assert L.brace_aggregate_update(FAKE_IN, 4, 100, 1, pr, eta, None, None) == E
    assert L.brace_aggregate_update(FAKE_IN, 4, 100, 1, None, eta, FAKE_OUT, None) == E
    assert L.brace_aggregate_update(FAKE_IN, 4, 100, 1, pr, eta, FAKE_IN + 40, None) == E
    assert L.brace_aggregate_update(FAKE_IN, 0, 100, 0, pr, eta, FAKE_OUT, None) == E
    assert L.brace_aggregate_update(FAKE_IN, 4, 0, 1, pr, eta, None, None) == B.BRACE_OK
    assert L.brace_aggregate_update_chunk(FAKE_IN, 4, 100, 1, 4, pr, eta, FAKE_OUT, None) == R
    assert L.brace_aggregate_update_chunk(FAKE_IN, 7, 3, 0, 6, pr, eta, FAKE_OUT, None) == B.BRACE_OK
    assert L.brace_expand_bits(None, 10, FAKE_OUT, None) == E
    assert L.brace_expand_bits(FAKE_IN, 10, None, None) == E
    assert L.brace_expand_bits(FAKE_IN + 2, 10, FAKE_OUT, None) == E
    assert L.brace_expand_bits(FAKE_IN, -1, FAKE_OUT, None) == E
    assert L.brace_expand_bits(None, 0, None, None) == B.BRACE_OK
    assert L.brace_apply_bits(FAKE_IN, 10, nan, FAKE_OUT, None) == E
    assert L.brace_apply_bits(FAKE_IN, 10, eta, None, None) == E
    assert L.brace_apply_bits(None, 0, eta, None, None) == B.BRACE_OK


def test_packed_entry_points_validate(L):
    E, R = B.BRACE_EINVAL, B.BRACE_ERANGE
    for d in (0, 1, 31, 32, 33, 64, 65, 1000, 25_000_000):
        assert B.brace_packed_row_words(d) == O.packed_row_words(d)
    p = B.make_params()
    pr = ctypes.byref(p)
    assert L.brace_quantize(None, 4, 100, 0, FAKE_OUT, 0, None) == E
    assert L.brace_quantize(FAKE_IN, 4, 100, 0, None, 0, None) == E
    assert L.brace_quantize(FAKE_IN, 4, 100, 0, FAKE_OUT + 8, 0, None) == E       # 16-byte rows
    assert L.brace_quantize(FAKE_IN, 4, 100, 50, FAKE_OUT, 0, None) == E          # ld < d
    assert L.brace_quantize(FAKE_IN, 4, 100, 0, FAKE_OUT, 4, None) == E           # pitch too small
    assert L.brace_quantize(FAKE_IN, 4, 100, 0, FAKE_OUT, 10, None) == E          # not a multiple of 4
    assert L.brace_quantize(FAKE_IN, 0, 100, 0, FAKE_OUT, 0, None) == E
    assert L.brace_quantize(FAKE_IN, 4, 100, 0, FAKE_IN + 64, 0, None) == E       # planes inside the matrix
    assert b"overlaps" in L.brace_last_error()
    assert L.brace_quantize(FAKE_IN, B.BRACE_MAX_CLIENTS + 1, 100, 0, FAKE_OUT, 0, None) == R
    assert L.brace_quantize(None, 4, 0, 0, None, 0, None) == B.BRACE_OK
    assert L.brace_vote_packed(FAKE_IN, 4, 100, 0, 1, None, FAKE_OUT, None) == E
    assert L.brace_vote_packed(None, 4, 100, 0, 1, pr, FAKE_OUT, None) == E
    assert L.brace_vote_packed(FAKE_IN, 4, 100, 0, 1, pr, None, None) == E          # no output
    assert L.brace_vote_packed(FAKE_IN, 4, 100, 0, 1, pr, FAKE_OUT + 4, None) == E  # out alignment
    assert L.brace_vote_packed(FAKE_IN, 4, 100, 6, 1, pr, FAKE_OUT, None) == E
    assert L.brace_vote_packed(FAKE_IN, 4, 100, 0, 5, pr, FAKE_OUT, None) == E      # f > n
    with_sums = B.make_params(sums_ptr=FAKE_OUT)
    assert L.brace_vote_packed(FAKE_IN, 4, 100, 0, 1, ctypes.byref(with_sums), FAKE_OUT, None) == E
    assert L.brace_vote_packed(None, 4, 0, 0, 1, pr, None, None) == B.BRACE_OK
    # chunk forms: the same checks plus the chunk index
    assert L.brace_vote_packed_chunk(FAKE_IN, 4, 100, 0, 1, 4, pr, FAKE_OUT, None) == R
    assert L.brace_vote_packed_chunk(FAKE_IN, 4, 100, 0, 1, -1, pr, FAKE_OUT, None) == R
    assert L.brace_vote_packed_chunk(None, 4, 100, 0, 1, 0, pr, FAKE_OUT, None) == E
    assert L.brace_vote_packed_chunk(FAKE_IN, 4, 100, 0, 1, 0, None, FAKE_OUT, None) == E
    assert L.brace_vote_packed_chunks(FAKE_IN, 4, 100, 0, 1, 2, 1, pr, FAKE_OUT, None) == R
    assert L.brace_vote_packed_chunks(FAKE_IN, 4, 100, 0, 1, 0, 5, pr, FAKE_OUT, None) == R
    assert L.brace_vote_packed_chunks(FAKE_IN, 0, 100, 0, 0, 0, 0, pr, FAKE_OUT, None) == E
    assert L.brace_vote_packed_chunks(FAKE_IN, 4, 100, 0, 9, 0, 4, pr, FAKE_OUT, None) == E   # f > n
    assert L.brace_vote_packed_chunks(None, 4, 100, 0, 1, 2, 2, pr, None, None) == B.BRACE_OK  # empty run
    assert L.brace_vote_packed_chunk(None, 8, 3, 0, 1, 5, pr, None, None) == B.BRACE_OK        # empty chunk (d < n)


def test_consensus_sums_validates(L):
    E, R = B.BRACE_EINVAL, B.BRACE_ERANGE
    p = B.make_params(5.0)
    pr = ctypes.byref(p)
    assert L.brace_consensus_sums(FAKE_IN, 4, 100, 0, None, FAKE_OUT, None) == E
    assert L.brace_consensus_sums(None, 4, 100, 0, pr, FAKE_OUT, None) == E
    assert L.brace_consensus_sums(FAKE_IN, 0, 100, 0, pr, FAKE_OUT, None) == E
    assert L.brace_consensus_sums(FAKE_IN, 4, -1, 0, pr, FAKE_OUT, None) == E
    assert L.brace_consensus_sums(FAKE_IN, 4, 100, 50, pr, FAKE_OUT, None) == E          # ld < d
    assert L.brace_consensus_sums(FAKE_IN, 4, 100, 0, pr, None, None) == E              # no output
    assert L.brace_consensus_sums(FAKE_IN + 1, 4, 100, 0, pr, FAKE_OUT, None) == E      # odd address
    assert L.brace_consensus_sums(FAKE_IN, 4, 100, 0, pr, FAKE_OUT + 2, None) == E
    assert L.brace_consensus_sums(FAKE_IN, 4, 100, 0, pr, FAKE_IN + 16, None) == E      # overlap
    assert L.brace_consensus_sums(FAKE_IN, B.BRACE_MAX_CLIENTS + 1, 100, 0, pr, FAKE_OUT, None) == R
    bad = B.make_params(float("nan"))
    assert L.brace_consensus_sums(FAKE_IN, 4, 100, 0, ctypes.byref(bad), FAKE_OUT, None) == E
    maj = B.make_params(0.0, rule=1)
    assert L.brace_consensus_sums(FAKE_IN, 4, 100, 0, ctypes.byref(maj), FAKE_OUT, None) == E
    with_sums = B.make_params(5.0, sums_ptr=FAKE_OUT)
    assert L.brace_consensus_sums(FAKE_IN, 4, 100, 0, ctypes.byref(with_sums), FAKE_OUT, None) == E
    assert L.brace_consensus_sums(None, 4, 0, 0, pr, None, None) == B.BRACE_OK


def test_absurd_sizes_are_range_errors_not_overflows(L):
    """Caller-supplied 64-bit sizes never reach arithmetic that could overflow."""
    R = B.BRACE_ERANGE
    p = B.make_params(5.0)
    pr = ctypes.byref(p)
    huge = 1 << 62
    assert L.brace_aggregate(FAKE_IN, 4, huge, 1, pr, FAKE_OUT, None) == R
    assert L.brace_aggregate(FAKE_IN, 32767, 1 << 40, 1, pr, FAKE_OUT, None) == R
    assert L.brace_aggregate_chunk(FAKE_IN, 4, huge, 1, 0, pr, FAKE_OUT, None) == R
    wide = B.make_params(5.0, ld=huge)
    assert L.brace_aggregate(FAKE_IN, 4, 100, 1, ctypes.byref(wide), FAKE_OUT, None) == R
    rp = B.BraceRarParams(ctypes.sizeof(B.BraceRarParams), 0, 0)
    assert L.brace_rar_aggregate(FAKE_IN, 4, huge, ctypes.byref(rp), FAKE_OUT, None) == R
    assert L.brace_aggregate_update(FAKE_IN, 4, huge, 1, pr, 0.1, FAKE_OUT, None) == R
    assert L.brace_quantize(FAKE_IN, 4, huge, 0, FAKE_OUT, 0, None) == R
    assert L.brace_vote_packed(FAKE_IN, 4, huge, 0, 1, pr, FAKE_OUT, None) == R
    assert L.brace_vote_packed(FAKE_IN, 4, (1 << 63) - 1, 0, 1, pr, FAKE_OUT, None) == R
    assert L.brace_vote_packed_chunk(FAKE_IN, 4, huge, 0, 1, 0, pr, FAKE_OUT, None) == R
    assert L.brace_consensus_sums(FAKE_IN, 4, huge, 0, pr, FAKE_OUT, None) == R
    assert L.brace_expand_bits(FAKE_IN, huge, FAKE_OUT, None) == R
    assert L.brace_apply_bits(FAKE_IN, huge, 0.1, FAKE_OUT, None) == R
    assert L.brace_packed_row_words((1 << 63) - 1) > 0
    assert L.brace_packed_row_words(-5) == 0


@pytest.mark.parametrize("m,n,d", [(32, 3, 3), (32, 100, 25_000_000), (8, 64, 100_000_000), (1, 1, 0),
                                   (64, 32767, 1 << 45), (16, 7, 1_000_003)])
def test_comm_cost_matches_the_closed_forms_of_the_oracle(L, m, n, d):
    for scheme, ref in ((B.BRACE_COST_SERVER_CLIENT, O.cost_sc), (B.BRACE_COST_RING_ALL_REDUCE, O.cost_rar),
                        (B.BRACE_COST_BRACE, O.cost_brace)):
        want = float(ref(m, n, d))
        got = B.brace_comm_cost(scheme, m, n, d)
        assert got == pytest.approx(want, rel=1e-15, abs=0.0)
    # BRACE sends less than plain ring-all-reduce whenever m > 1 (Sec. 3, cost paragraph)
    if m > 1 and n > 1 and d > 0:
        assert B.brace_comm_cost(B.BRACE_COST_BRACE, m, n, d) < \
            B.brace_comm_cost(B.BRACE_COST_RING_ALL_REDUCE, m, n, d)


def test_comm_cost_validates(L):
    v = ctypes.c_double()
    E = B.BRACE_EINVAL
    assert L.brace_comm_cost(0, 32, 4, 100, None) == E
    assert L.brace_comm_cost(3, 32, 4, 100, ctypes.byref(v)) == E
    assert L.brace_comm_cost(-1, 32, 4, 100, ctypes.byref(v)) == E
    assert L.brace_comm_cost(0, 0, 4, 100, ctypes.byref(v)) == E
    assert L.brace_comm_cost(0, 65, 4, 100, ctypes.byref(v)) == E
    assert L.brace_comm_cost(0, 32, 0, 100, ctypes.byref(v)) == E
    assert L.brace_comm_cost(0, 32, 4, -1, ctypes.byref(v)) == E


def test_one_bit_entry_points_validate(L):
    E, R = B.BRACE_EINVAL, B.BRACE_ERANGE
    p = B.make_params(5.0)
    pr = ctypes.byref(p)
    for d in (0, 1, 31, 32, 33, 127, 128, 129, 1000, 25_000_000):
        assert L.brace_1bit_row_words(d) == O.vote_plane_row_words(d)
    assert L.brace_1bit_row_words(-3) == 0 and L.brace_1bit_row_words((1 << 63) - 1) > 0
    assert L.brace_quantize_1bit(FAKE_IN, 4, 100, 0, 0, FAKE_OUT, 0, None) == E       # zeros abstain
    assert b"two-plane" in L.brace_last_error()
    assert L.brace_quantize_1bit(FAKE_IN, 4, 100, 0, 2, FAKE_OUT, 0, None) == E
    assert L.brace_quantize_1bit(None, 4, 100, 0, 1, FAKE_OUT, 0, None) == E
    assert L.brace_quantize_1bit(FAKE_IN, 4, 100, 0, 1, None, 0, None) == E
    assert L.brace_quantize_1bit(FAKE_IN, 4, 100, 0, 1, FAKE_OUT + 8, 0, None) == E
    assert L.brace_quantize_1bit(FAKE_IN, 4, 100, 50, 1, FAKE_OUT, 0, None) == E
    assert L.brace_quantize_1bit(FAKE_IN, 4, 100, 0, 1, FAKE_OUT, 2, None) == E
    assert L.brace_quantize_1bit(FAKE_IN, 4, 100, 0, 1, FAKE_OUT, 6, None) == E
    assert L.brace_quantize_1bit(FAKE_IN, 4, 100, 0, 1, FAKE_IN + 64, 0, None) == E   # overlap
    assert L.brace_quantize_1bit(FAKE_IN, 0, 100, 0, 1, FAKE_OUT, 0, None) == E
    assert L.brace_quantize_1bit(FAKE_IN, B.BRACE_MAX_CLIENTS + 1, 100, 0, 1, FAKE_OUT, 0, None) == R
    assert L.brace_quantize_1bit(FAKE_IN, 4, 1 << 62, 0, 1, FAKE_OUT, 0, None) == R
    assert L.brace_quantize_1bit(None, 4, 0, 0, -1, None, 0, None) == B.BRACE_OK
    assert L.brace_vote_1bit(FAKE_IN, 4, 100, 0, 1, None, FAKE_OUT, None) == E
    assert L.brace_vote_1bit(None, 4, 100, 0, 1, pr, FAKE_OUT, None) == E
    assert L.brace_vote_1bit(FAKE_IN, 4, 100, 0, 1, pr, None, None) == E
    assert L.brace_vote_1bit(FAKE_IN, 4, 100, 0, 1, pr, FAKE_OUT + 4, None) == E
    assert L.brace_vote_1bit(FAKE_IN, 4, 100, 2, 1, pr, FAKE_OUT, None) == E
    assert L.brace_vote_1bit(FAKE_IN, 4, 100, 0, 5, pr, FAKE_OUT, None) == E
    assert L.brace_vote_1bit(FAKE_IN, 4, 1 << 62, 0, 1, pr, FAKE_OUT, None) == R
    maj = B.make_params(0.0, rule=1)
    assert L.brace_vote_1bit(FAKE_IN, 4, 100, 0, 1, ctypes.byref(maj), FAKE_OUT, None) == E
    assert L.brace_vote_1bit(None, 4, 0, 0, 1, pr, None, None) == B.BRACE_OK
    assert L.brace_vote_1bit_chunks(FAKE_IN, 4, 100, 0, 1, 2, 1, pr, FAKE_OUT, None) == R
    assert L.brace_vote_1bit_chunks(FAKE_IN, 4, 100, 0, 1, 0, 5, pr, FAKE_OUT, None) == R
    assert L.brace_vote_1bit_chunks(None, 4, 100, 0, 1, 0, 2, pr, FAKE_OUT, None) == E
    assert L.brace_vote_1bit_chunks(None, 4, 100, 0, 1, 2, 2, pr, None, None) == B.BRACE_OK


def test_rar_aggregate_rejects_invalid_arguments(L):
    def call(inp=FAKE_IN, n=4, d=100, mean=0, ld=0, out=FAKE_OUT, size=None, chunk=None, order=0,
             reserved=0):
        p = B.BraceRarParams(ctypes.sizeof(B.BraceRarParams) if size is None else size, mean, ld,
                             order, reserved)
        if chunk is None:
            return L.brace_rar_aggregate(inp, n, d, ctypes.byref(p), out, None)
        return L.brace_rar_aggregate_chunk(inp, n, d, chunk, ctypes.byref(p), out, None)
    E, R = B.BRACE_EINVAL, B.BRACE_ERANGE
    assert ctypes.sizeof(B.BraceRarParams) == 24
    assert L.brace_rar_aggregate(FAKE_IN, 4, 100, None, FAKE_OUT, None) == E
    assert call(size=8) == E
    assert call(size=16) == E                 # the layout before `order` was added
    assert call(order=2) == E and call(order=-1) == E and call(order=1, reserved=1) == E
    for order in (0, 1):                      # both orders run the same checks
        assert call(order=order, d=0) == B.BRACE_OK
        assert call(order=order, out=FAKE_IN + 40) == E
        assert call(order=order, chunk=4) == R
        assert call(order=order, n=7, d=3, chunk=6) == B.BRACE_OK
    assert call(n=0) == E
    assert call(n=B.BRACE_MAX_CLIENTS + 1) == R
    assert call(d=-1) == E
    assert call(mean=2) == E
    assert call(ld=50) == E
    assert call(inp=None) == E
    assert call(out=None) == E
    assert call(inp=FAKE_IN + 1) == E
    assert call(out=FAKE_IN + 40) == E
    assert call(chunk=4) == R
    assert call(d=0) == B.BRACE_OK
    assert call(d=0, inp=None, out=None) == B.BRACE_OK
    assert call(n=7, d=3, chunk=6) == B.BRACE_OK        # empty chunk, nothing launched


def test_tuning_roundtrip_and_validation(L):
    B.brace_reset_tuning()
    base = B.brace_get_tuning()
    assert set(base) == {"vec", "cols", "unroll", "nontemporal", "pipeline", "split_writes",
                         "rowsplit", "stage_writes"}
    B.brace_set_tuning(vec=2, cols=4, unroll=8, nontemporal=0, pipeline=0, split_writes=2,
                       rowsplit=2, stage_writes=1)
    assert B.brace_get_tuning() == {"vec": 2, "cols": 4, "unroll": 8, "nontemporal": 0,
                                    "pipeline": 0, "split_writes": 2, "rowsplit": 2,
                                    "stage_writes": 1}
    with pytest.raises(B.BraceError):
        B.brace_set_tuning(stage_writes=3)
    with pytest.raises(B.BraceError):
        B.brace_set_tuning(rowsplit=3)
    with pytest.raises(B.BraceError):
        B.brace_set_tuning(split_writes=3)
    with pytest.raises(B.BraceError):
        B.brace_set_tuning(vec=3)
    with pytest.raises(B.BraceError):
        B.brace_set_tuning(cols=3)
    with pytest.raises(B.BraceError):
        B.brace_set_tuning(unroll=5)
    B.brace_reset_tuning()
    assert B.brace_get_tuning() == base


def test_binding_has_no_fallback_path():
    # The product path must not reach the oracle or any CPU implementation.
    pkg = os.path.join(ROOT, "paper_2501_17392_amd")
    for fn in os.listdir(pkg):
        if fn.endswith(".py"):
            text = open(os.path.join(pkg, fn)).read()
            assert "import oracle" not in text and "from oracle" not in text, fn
    text = open(os.path.join(ROOT, "oracle", "brace_oracle.py")).read()
    assert "paper_2501_17392_amd" not in text
