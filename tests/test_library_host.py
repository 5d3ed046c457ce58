"""The library's host side against the oracle (CPU only, no GPU calls).

The host encoder of libmacko is a separate implementation (two parallel passes
and a closed-form padding count); it must agree with the oracle byte for byte.
"""
import ctypes
import os
import re
import subprocess

import numpy as np
import pytest

import oracle
import workloads as wl

M = pytest.importorskip("paper_2511_13061_amd")
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def same_encoding(m, enc):
    v, d, r = m.host_buffers()
    assert v.dtype == np.uint16 and d.dtype == np.uint8 and r.dtype == np.uint32
    assert np.array_equal(v, enc.values)
    assert np.array_equal(d, enc.deltas)
    assert np.array_equal(r, enc.row_ptr)


def same_report(rep, enc, W, b_delta=4):
    assert (rep.rows, rep.cols) == W.shape
    assert rep.nnz == enc.nnz and rep.pad_nnz == enc.pad_nnz and rep.alloc_nnz == enc.alloc_nnz
    assert rep.padding_entries == enc.padding_entries
    assert rep.values_bytes == enc.values_bytes and rep.deltas_bytes == enc.deltas_bytes
    assert rep.rowptr_bytes == enc.rowptr_bytes and rep.total_bytes == enc.total_bytes
    assert rep.dense_bytes == enc.dense_bytes
    ent = np.diff(enc.row_ptr.astype(np.int64))
    assert rep.empty_rows == int((ent == 0).sum())
    assert rep.max_row_entries == (int(ent.max()) if ent.size else 0)
    assert rep.b_val == 16 and rep.b_delta == b_delta
    if W.size:
        d = enc.nnz / W.size
        cf = oracle.closed_forms
        assert rep.density == pytest.approx(d, abs=1e-15)
        assert rep.effd == pytest.approx(enc.effd, rel=1e-14)
        assert rep.effd_best == pytest.approx(cf.effd_macko_best(d, b_delta=b_delta), rel=1e-13)
        assert rep.effd_worst == pytest.approx(cf.effd_macko_worst(d, b_delta=b_delta), rel=1e-13)
        assert rep.effd_expected == pytest.approx(cf.effd_macko_expected(d, b_delta=b_delta), rel=1e-12)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "macko.h")).read()
    declared = set(re.findall(r"MACKO_API\s+[\w\s\*]+?\b(macko_\w+)\s*\(", header))
    assert declared == set(M.binding.EXPORTED_SYMBOLS)
    lib = ctypes.CDLL(M.library_path())
    for name in declared:
        assert hasattr(lib, name), name


def test_header_is_plain_c_and_cpp(tmp_path):
    """The boundary is a C ABI: include/macko.h must compile as C99 and as C++11, pedantic, without warnings."""
    c = tmp_path / "use.c"
    c.write_text('#include "macko.h"\nint main(void) { macko_report_t r; macko_handle_t h = 0; (void)r; (void)h; return 0; }\n')
    inc = os.path.join(ROOT, "include")
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-I", inc, str(c)])
    cpp = tmp_path / "use.cpp"
    cpp.write_text(c.read_text())
    subprocess.check_call(["g++", "-std=c++11", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-I", inc, str(cpp)])


CASES = [
    ("c1", lambda: wl.config1().W),
    ("bern_sparse", lambda: wl.bernoulli(97, 1531, 0.03, 1.0, 5, 1)),
    ("bern_half", lambda: wl.bernoulli(130, 777, 0.5, 0.02, 5, 2)),
    ("dense", lambda: wl.bernoulli(33, 257, 1.0, 0.02, 5, 3)),
    ("c4", lambda: wl.config4(rows=96, cols=1200).W),
    ("c4b", lambda: wl.config4b(rows=40, cols=992).W),
    ("one_col", lambda: wl.bernoulli(50, 1, 0.5, 1.0, 5, 4)),
    ("wide_empty", lambda: np.zeros((9, 4000), dtype=np.uint16)),
]


@pytest.mark.parametrize("name,make", CASES, ids=[c[0] for c in CASES])
def test_host_encoder_is_bit_exact_against_the_oracle(name, make):
    W = make()
    enc = oracle.encode(W)
    rep_holder = M.encode(W)
    same_encoding(rep_holder, enc)
    same_report(rep_holder.report, enc, W)
    assert np.array_equal(rep_holder.decode(), oracle.decode(enc))
    rep_holder.destroy()


@pytest.mark.parametrize("b_delta", [1, 2, 8])
@pytest.mark.parametrize("name,make", CASES, ids=[c[0] for c in CASES])
def test_host_encoder_other_code_widths_bit_exact_against_the_oracle(name, make, b_delta):
    """macko_encode_ex: 1-, 2- and 8-bit codes (Section 4.1 allows exactly 1, 2, 4, 8)."""
    W = make()
    enc = oracle.encode(W, b_delta)
    m = M.encode(W, b_delta)
    same_encoding(m, enc)
    same_report(m.report, enc, W, b_delta)
    assert np.array_equal(m.decode(), oracle.decode(enc))
    vb, db, rb = m.device_bytes()
    assert (vb, db, rb) == (enc.values_bytes, enc.deltas_bytes, enc.rowptr_bytes)
    m.destroy()


def test_worked_example_of_section_4_1_through_the_library():
    """The paper's row (values 1..4 at 1-based columns 2, 5, 12, 13) with 2-bit codes stores
    values [1, 2, 0, 3, 4] with deltas [2, 3, 4, 3, 1]."""
    one = np.float16([1, 2, 3, 4]).view(np.uint16)
    W = np.zeros((1, 16), dtype=np.uint16)
    W[0, [1, 4, 11, 12]] = one
    m = M.encode(W, 2)
    v, d, r = m.host_buffers()
    assert r.tolist() == [0, 5]
    assert v[:5].tolist() == [one[0], one[1], 0, one[2], one[3]]
    codes = [(int(d[k // 4]) >> (2 * (k % 4))) & 3 for k in range(5)]
    assert [c + 1 for c in codes] == [2, 3, 4, 3, 1]
    assert m.report.padding_entries == 1 and m.report.alloc_nnz == 64


def test_code_width_argument_is_validated():
    lib = M.load_library()
    W = np.ones((2, 2), dtype=np.uint16)
    h = ctypes.c_void_p(5)
    for bad in (0, 3, 5, 16, -4):
        assert lib.macko_encode_ex(W.ctypes.data, 2, 2, 2, bad, ctypes.byref(h), None) == -1
        assert h.value is None
        assert lib.macko_wrap_device_ex(2, 2, 4, bad, 256, 256, 256, ctypes.byref(h)) == -1
    m = M.encode(W, 2)
    assert lib.macko_spmm(m._h, 2, 16, 2, 16, 2, None) == -5    # not bound: refused before any device work


def test_special_bit_patterns_and_strided_input():
    W = np.zeros((6, 100), dtype=np.uint16)
    W[0, 3] = 0x8000      # -0 dropped
    W[0, 99] = 0x0001     # subnormal kept, long gap
    W[1, 0] = 0x7C00
    W[2, 50] = 0xFE00
    W[5, 17] = 0x8001
    big = np.zeros((6, 128), dtype=np.uint16)
    big[:, :100] = W
    m = M.encode(big[:, :100])          # ld = 128 > cols
    same_encoding(m, oracle.encode(W))
    canon = W.copy(); canon[0, 3] = 0
    assert np.array_equal(m.decode(), canon)


def test_empty_shapes_and_error_codes():
    lib = M.load_library()
    for shape in [(0, 5), (5, 0), (0, 0)]:
        m = M.encode(np.zeros(shape, dtype=np.uint16))
        assert m.report.pad_nnz == 0 and m.report.alloc_nnz == 0
        v, d, r = m.host_buffers()
        assert r.tolist() == [0] * (shape[0] + 1) and v.size == 0 and d.size == 0
    h = ctypes.c_void_p(123)
    W = np.ones((2, 2), dtype=np.uint16)
    assert lib.macko_encode(W.ctypes.data, 2, 2, 1, ctypes.byref(h), None) == -1   # ld < cols
    assert h.value is None
    assert lib.macko_encode(None, 2, 2, 2, ctypes.byref(h), None) == -1
    assert lib.macko_encode(W.ctypes.data, -1, 2, 2, ctypes.byref(h), None) == -1
    assert lib.macko_encode(W.ctypes.data, 2, 2, 2, None, None) == -1
    m = M.encode(W)
    # not bound: device operations are refused without touching the GPU
    assert lib.macko_spmv(m._h, 16, 16, None) == -5
    assert lib.macko_fetch_device(m._h, 16, 16, 16) == -5
    assert M.status_string(-5) == "handle has no device buffers"
    assert M.status_string(0) == "ok"
    with pytest.raises(M.MackoError):
        M.set_tuning("no_such_knob", 1)
    with pytest.raises(M.MackoError):
        M.set_tuning("spmv_block", 100)
    M.set_tuning("spmv_block", 256)
    assert M.get_tuning("spmv_block") == 256
    M.set_tuning("spmv_block", 0)
    for bad in (4, 100, 1024):                            # a power of two from 8 to 512
        with pytest.raises(M.MackoError):
            M.set_tuning("spmv_step_align", bad)
    M.set_tuning("spmv_step_align", 128)
    assert M.get_tuning("spmv_step_align") == 128
    M.set_tuning("spmv_step_align", 0)
    lib.macko_destroy(None)


def test_padding_bound_reported_for_llama_like_rows():
    W = wl.half_row_matrix(64, 4096, 77)
    m = M.encode(W)
    r = m.report
    assert r.nnz == 64 * 2048 and r.density == 0.5
    assert r.effd_best <= r.effd <= r.effd_worst
    assert r.padding_entries <= 64 * 4096 * 0.5 / 16


def test_kernels_use_no_scratch_memory(tmp_path):
    """No kernel may spill registers or keep a run-time-indexed array in scratch memory: a scratch
    store per step costs more HBM bandwidth than the format saves (this happened to the 8-bit decode)."""
    import shutil
    import subprocess
    from paper_2511_13061_amd import build as B
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("no hipcc")
    flags = [f for f in B.HIPCC_FLAGS if f not in ("-fPIC",)]
    for src in (s for s in B.SOURCES if s.endswith(".hip")):
        out = tmp_path / (src + ".s")
        subprocess.check_call([hipcc, *flags, "-I", os.path.join(ROOT, "include"), "-I", B.CSRC, "-x", "hip",
                               "--cuda-device-only", "-S", "-o", str(out), os.path.join(B.CSRC, src)],
                              stderr=subprocess.DEVNULL)
        text = out.read_text()
        assert ".amdhsa_kernel" in text, src
        assert not re.search(r"^\s*scratch_(load|store)", text, re.M), f"{src}: scratch memory access"
        assert not re.search(r"\.private_segment_fixed_size:\s*[1-9]", text), f"{src}: private segment in use"
        # (scalar registers parked in lanes of a vector register are not memory: only vector spills count)
        assert not re.search(r"\.vgpr_spill_count:\s*[1-9]", text), f"{src}: vector register spills"


def test_launch_planner_covers_every_row_exactly_once(tmp_path):
    """Host logic of the launch planner: tests/planner_check.cpp replays, for 3000 random groups of
    matrices and both launch regimes, the row assignment the kernels derive from a plan."""
    import shutil
    import subprocess
    from paper_2511_13061_amd import build as B
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("no hipcc")
    exe = tmp_path / "planner_check"
    subprocess.check_call([hipcc, "-std=c++17", "-O1", "-I", os.path.join(ROOT, "include"), "-I", B.CSRC,
                           os.path.join(ROOT, "tests", "planner_check.cpp"), "-o", str(exe)],
                          stderr=subprocess.DEVNULL)
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0 and out.stdout.startswith("ok"), out.stdout + out.stderr


def test_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The library's host translation unit (encoders for every code and value width, decoders, storage
    report, argument checks) linked with stand-ins for the GPU launchers and run under ASan + UBSan on
    random, ragged, strided, empty and overflowing inputs (tests/host_sanitizer_check.cpp)."""
    import shutil
    import subprocess
    from paper_2511_13061_amd import build as B
    if not shutil.which("g++") or not os.path.exists("/opt/rocm/lib/libamdhip64.so"):
        pytest.skip("needs g++ and the HIP runtime library to link against")
    exe = tmp_path / "host_sanitizer_check"
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=undefined", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
                           "-I", os.path.join(ROOT, "include"), "-I", B.CSRC,
                           os.path.join(ROOT, "tests", "host_sanitizer_check.cpp"),
                           os.path.join(ROOT, "tests", "host_sanitizer_stubs.cpp"),
                           os.path.join(B.CSRC, "macko_host.cpp"), "-o", str(exe),
                           "-L/opt/rocm/lib", "-lamdhip64", "-lpthread", "-Wl,-rpath,/opt/rocm/lib"],
                          stderr=subprocess.DEVNULL)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=600, env=env)
    assert out.returncode == 0 and out.stdout.strip().endswith("ok"), out.stdout[-2000:] + out.stderr[-4000:]


# ------------------------------------------------------------------ 8-bit values (host side)

@pytest.mark.parametrize("shape,density", [((64, 512), 0.5), ((33, 1031), 0.07), ((5, 40), 1.0), ((300, 2000), 0.3)])
def test_host_encoder_for_8_bit_values_is_bit_exact_against_the_oracle(shape, density):
    rng = np.random.default_rng(shape[0])
    W = rng.integers(0, 256, size=shape, dtype=np.uint8)
    W[rng.random(shape) >= density] = 0
    W[0, :] = 0
    W[1, 0] = 0x80                                         # -0 is a zero
    W[2, shape[1] - 1] = 0xFF                              # a NaN pattern is a value like any other
    enc = oracle.encode8(W, 4)
    m = M.encode_fp8(W)
    v, d, r = m.host_buffers()
    assert v.dtype == np.uint8
    assert np.array_equal(v, enc.values) and np.array_equal(d, enc.deltas) and np.array_equal(r, enc.row_ptr)
    rep = m.get_report()
    assert (rep.b_val, rep.b_delta, rep.nnz, rep.pad_nnz, rep.alloc_nnz) == (8, 4, enc.nnz, enc.pad_nnz, enc.alloc_nnz)
    assert (rep.values_bytes, rep.deltas_bytes, rep.total_bytes, rep.dense_bytes) == \
        (enc.values_bytes, enc.deltas_bytes, enc.total_bytes, enc.dense_bytes)
    assert rep.effd == pytest.approx(enc.effd, rel=1e-12)
    dd = enc.nnz / (shape[0] * shape[1])
    assert rep.effd_best == pytest.approx(oracle.closed_forms.effd_macko_best(dd, 8, 4), rel=1e-12)
    assert rep.effd_worst == pytest.approx(oracle.closed_forms.effd_macko_worst(dd, 8, 4), rel=1e-12)
    assert rep.effd_expected == pytest.approx(oracle.closed_forms.effd_macko_expected(dd, 8, 4), rel=1e-12)
    assert np.array_equal(m.decode(), oracle.decode8(enc))
    assert m.device_bytes() == (enc.alloc_nnz, enc.alloc_nnz // 2, 4 * (shape[0] + 1))
    # strided input
    wide = np.zeros((shape[0], shape[1] + 7), dtype=np.uint8)
    wide[:, :shape[1]] = W
    v2, d2, r2 = M.encode_fp8(wide[:, :shape[1]]).host_buffers()
    assert np.array_equal(v2, enc.values) and np.array_equal(d2, enc.deltas) and np.array_equal(r2, enc.row_ptr)


def test_8_bit_handles_refuse_what_they_do_not_support():
    lib = M.load_library()
    W = np.full((4, 64), 0x38, dtype=np.uint8)
    m8 = M.encode_fp8(W)
    m16 = M.encode(np.full((4, 64), 0x3C00, dtype=np.uint16))
    buf16 = np.zeros((4, 64), dtype=np.uint16)
    buf8 = np.zeros((4, 64), dtype=np.uint8)
    assert lib.macko_decode(m8._h, buf16.ctypes.data, 64) == -3            # MACKO_E_UNSUPPORTED
    assert lib.macko_decode_fp8(m16._h, buf8.ctypes.data, 64) == -3
    p = ctypes.c_void_p()
    assert lib.macko_host_values_fp8(m16._h, ctypes.byref(p)) == -3
    assert lib.macko_host_buffers(m8._h, ctypes.byref(p), None, None) == -3
    assert lib.macko_encode_fp8(None, 4, 64, 64, ctypes.byref(p), None) == -1
    assert lib.macko_encode_fp8(W.ctypes.data, 4, 64, 63, ctypes.byref(p), None) == -1
    empty = M.encode_fp8(np.zeros((0, 16), dtype=np.uint8))
    assert empty.get_report().pad_nnz == 0


def test_storage_by_code_width_equals_the_oracles_encodings():
    """Bytes per code width counted without encoding (Section 4.2 / Appendix C) against the oracle's
    encodings at each width, and the choice: 1 bit for dense rows, 2 bits around 40 %, 4 bits at
    70 %, 8 bits at 97 % sparsity (the ranges of Appendix C)."""
    cases = {
        "dense": (wl.bernoulli(40, 1031, 1.0, 0.02, 91, 1), 1),
        "sparsity40": (wl.bernoulli(64, 3000, 0.6, 0.02, 91, 2), 2),
        "sparsity70": (wl.bernoulli(64, 3000, 0.3, 0.02, 91, 3), 4),
        "sparsity97": (wl.bernoulli(300, 9000, 0.03, 1.0, 91, 4), 8),
        "worked_example": (None, None),
    }
    for name, (W, want_best) in cases.items():
        if W is None:
            W = np.zeros((3, 12), dtype=np.uint16)
            W[0, [0, 4, 11]] = 0x3C00
            W[2, 7] = 0x4000
        table, best = M.storage_by_code_width(W)
        for b in (1, 2, 4, 8):
            assert table[b] == oracle.encode(W, b).total_bytes, (name, b)
        assert table[best] == min(table.values())
        if want_best is not None:
            assert best == want_best, (name, table)
    # empty matrix: only the row pointers (and a tie, which goes to 4 bits)
    table, best = M.storage_by_code_width(np.zeros((5, 0), dtype=np.uint16))
    assert set(table.values()) == {4 * 6} and best == 4
    lib = M.load_library()
    out = (ctypes.c_int64 * 4)()
    assert lib.macko_storage_by_code_width(None, 2, 2, 2, out, None) == -1
    assert lib.macko_storage_by_code_width(W.ctypes.data, 3, 12, 4, out, None) == -1       # ld < cols
