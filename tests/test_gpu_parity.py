"""GPU parity: the HIP path (through the C ABI) against the CPU oracle.

Encodings must match the oracle byte for byte.  Every y_i must satisfy
|y_gpu - y_fp64| <= 1e-2 * sum_j |w_ij x_j| + 1e-3, with y_fp64 the dense
product by definition (Appendix A of the paper) computed by the oracle.
"""
import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
M = pytest.importorskip("paper_2511_13061_amd")

REL_TOL = 1e-2
ABS_TOL = 1e-3


@pytest.fixture(scope="module", autouse=True)
def _need_gpu_and_library():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    M.load_library()          # raises if libmacko.so is missing: no fallback
    yield
    for knob in ("spmv_kernel", "spmv_lanes", "spmv_block", "spmv_rows_per_wg", "spmv_ring", "spmv_resident",
                 "spmv_wgs_per_cu", "spmv_resident_steps", "spmv_steps_per_wave", "spmv_step_align", "gemv_block", "gemv_rows_per_wg", "gemv_ring", "gemv_resident",
                 "gemv_wgs_per_cu"):
        M.set_tuning(knob, 0)


def to_dev(a_u16):
    return torch.from_numpy(np.ascontiguousarray(a_u16).view(np.float16)).cuda()


def check_y(y_dev, W, x, what=""):
    y64, s64 = oracle.dense_matvec(W, x)
    y = y_dev.float().cpu().numpy().astype(np.float64)
    assert y.shape == y64.shape
    assert np.isfinite(y).all(), what
    err = np.abs(y - y64)
    bound = REL_TOL * s64 + ABS_TOL
    worst = int(np.argmax(err - bound))
    assert (err <= bound).all(), (
        f"{what}: row {worst}: |{y[worst]} - {y64[worst]}| = {err[worst]} > {bound[worst]}")
    # the tolerance is loose; fp32 accumulation should in fact sit well inside it
    return float(np.max(err / bound))


def spmv_case(W, x, b_delta=4, **knobs):
    for k, v in knobs.items():
        M.set_tuning(k, v)
    try:
        m = M.encode(W, b_delta).to_device()
        y = m.spmv(to_dev(x))
        torch.cuda.synchronize()
    finally:
        for k in knobs:
            M.set_tuning(k, 0)
    return y


def assert_same_encoding(arrays, enc):
    v, d, r = arrays
    assert np.array_equal(r, enc.row_ptr)
    assert np.array_equal(v, enc.values)
    assert np.array_equal(d, enc.deltas)


# ------------------------------------------------------------------ small and ragged

SMALL = {
    "c1_512": lambda: (wl.config1().W, wl.config1().x),
    "ragged_777": lambda: (wl.bernoulli(301, 777, 0.5, 0.02, 9, 1), wl.x_vector(777, 9, 1)),
    "long_rows_5000": lambda: (wl.bernoulli(70, 5000, 0.6, 0.02, 9, 2), wl.x_vector(5000, 9, 2)),
    "very_sparse": lambda: (wl.bernoulli(200, 3000, 0.02, 1.0, 9, 3), wl.x_vector(3000, 9, 3)),
    "dense": lambda: (wl.bernoulli(100, 1031, 1.0, 0.02, 9, 4), wl.x_vector(1031, 9, 4)),
    "c4_small": lambda: (wl.config4(rows=256, cols=2048).W, wl.config4(rows=256, cols=2048).x),
    "c4b_small": lambda: (wl.config4b(rows=128, cols=2048).W, wl.config4b(rows=128, cols=2048).x),
    "one_row": lambda: (wl.bernoulli(1, 9000, 0.5, 0.02, 9, 5), wl.x_vector(9000, 9, 5)),
    "one_col": lambda: (wl.bernoulli(300, 1, 0.5, 1.0, 9, 6), wl.x_vector(1, 9, 6)),
}

VARIANTS = {
    "auto": {},
    "sub16": {"spmv_kernel": 1, "spmv_lanes": 16},
    "sub32": {"spmv_kernel": 1, "spmv_lanes": 32},
    "sub64": {"spmv_kernel": 1, "spmv_lanes": 64},
    "wave_row": {"spmv_kernel": 2},
    "wave_row_b256_r5": {"spmv_kernel": 2, "spmv_block": 256, "spmv_rows_per_wg": 5},
    "wave_row_b1024_r700": {"spmv_kernel": 2, "spmv_block": 1024, "spmv_rows_per_wg": 700},
    "wave_row_b64_r200": {"spmv_kernel": 2, "spmv_block": 64, "spmv_rows_per_wg": 200},
    "wave_row_b256_r37": {"spmv_kernel": 2, "spmv_block": 256, "spmv_rows_per_wg": 37},
    "wave_row_b128_r63": {"spmv_kernel": 2, "spmv_block": 128, "spmv_rows_per_wg": 63},
    # every step of a row on a multiple of 64 / 256 / 512 stored entries (lanes before the row cleared)
    "wave_row_align64": {"spmv_kernel": 2, "spmv_step_align": 64},
    "wave_row_align256_b256_r37": {"spmv_kernel": 2, "spmv_step_align": 256, "spmv_block": 256, "spmv_rows_per_wg": 37},
    "wave_row_align512": {"spmv_kernel": 2, "spmv_step_align": 512},
}


@pytest.mark.parametrize("variant", list(VARIANTS))
@pytest.mark.parametrize("case", list(SMALL))
def test_spmv_small_cases_all_kernels(case, variant):
    W, x = SMALL[case]()
    y = spmv_case(W, x, **VARIANTS[variant])
    check_y(y, W, x, f"{case}/{variant}")


def test_spmv_empty_rows_mixed_with_full_rows_and_row_boundaries_inside_chunks():
    rng = np.random.default_rng(5)
    C = 4096
    W = wl.bernoulli(400, C, 0.5, 0.02, 11, 1)
    W[rng.choice(400, 120, replace=False)] = 0           # empty rows, some adjacent
    W[10:30] = 0
    W[395:] = 0                                          # trailing empty rows
    # rows with 1..9 entries so that several rows share one 8-entry chunk
    for r in range(40, 60):
        W[r] = 0
        cols = rng.choice(C, size=(r - 39) % 10 + 1, replace=False)
        W[r, cols] = wl.normal_f16(cols.size, 1.0, 11, r, nonzero=True)
    x = wl.x_vector(C, 11, 1)
    for variant in ("auto", "wave_row", "sub16", "wave_row_b64_r200", "wave_row_b256_r37", "wave_row_b128_r63",
                    "wave_row_align64", "wave_row_align256_b256_r37", "wave_row_align512"):
        y = spmv_case(W, x, **VARIANTS[variant])
        check_y(y, W, x, variant)
        assert (y[10:30] == 0).all() and (y[395:] == 0).all()


@pytest.mark.parametrize("b_delta", [1, 4, 8])
def test_aligned_steps_with_rows_starting_at_chosen_offsets(b_delta):
    """Rows whose first k columns are non-zero (no padding), so that every row starts at a known
    entry: multiples of the step alignment, one entry after, eight after, one before; rows of one
    entry, empty rows and rows of exactly one and two steps between them.  Each alignment of the
    wave-per-row kernel, and the choice it makes by itself."""
    C = 4096
    lengths = [512, 256, 1, 7, 8, 9, 247, 248, 1, 255, 256, 257, 0, 0, 3, 1024, 511, 513, 2048, 64, 63, 65,
               4096, 1, 4095, 0, 1536, 8, 504, 16, 1000, 3000, 2, 510, 4096, 4096, 5, 251]
    W = np.zeros((len(lengths), C), dtype=np.uint16)
    for r, n in enumerate(lengths):
        if n:
            W[r, :n] = wl.normal_f16(n, 1.0, 77, r, nonzero=True)
    x = wl.x_vector(C, 77, 1)
    enc = oracle.encode(W, b_delta)
    assert enc.pad_nnz == sum(lengths) and list(np.diff(enc.row_ptr.astype(np.int64))) == lengths
    for knobs in ({}, {"spmv_kernel": 2}, {"spmv_kernel": 2, "spmv_step_align": 64},
                  {"spmv_kernel": 2, "spmv_step_align": 256, "spmv_block": 128, "spmv_rows_per_wg": 5},
                  {"spmv_kernel": 2, "spmv_step_align": 512, "spmv_block": 64, "spmv_rows_per_wg": 38},
                  {"spmv_kernel": 2, "spmv_step_align": 512, "spmv_ring": 4},
                  {"spmv_kernel": 2, "spmv_step_align": 16, "spmv_ring": 3}):
        y = spmv_case(W, x, b_delta, **knobs)
        check_y(y, W, x, f"b{b_delta}/{knobs}")
        assert y[12] == 0 and y[13] == 0 and y[25] == 0


def test_random_matrices_with_random_launch_knobs():
    """Forty seeded draws of shape, density, code width and launch knobs (kernel, block, rows per
    workgroup, resident round, ring depth, step alignment): the planner has to turn every
    combination into a launch that computes each row exactly once."""
    rng = np.random.default_rng(20251113)
    for case in range(40):
        rows = int(rng.integers(1, 400))
        cols = int(rng.choice([1, 7, 64, 500, 1031, 2048, 4096, 6000, 9000]))
        dens = float(rng.choice([0.02, 0.1, 0.3, 0.5, 0.8, 1.0]))
        b_delta = int(rng.choice([1, 2, 4, 8]))
        W = wl.bernoulli(rows, cols, dens, 0.05, 700 + case, 1)
        if rows > 5:
            W[rng.choice(rows, rows // 5, replace=False)] = 0     # empty rows
        x = wl.x_vector(cols, 700 + case, 2)
        block = int(rng.choice([0, 64, 128, 192, 256, 512, 704, 1024]))
        knobs = {"spmv_kernel": int(rng.choice([0, 2, 2, 2])), "spmv_block": block,
                 "spmv_step_align": int(rng.choice([0, 8, 16, 32, 64, 128, 256, 512])),
                 "spmv_ring": int(rng.choice([0, 2, 3, 4])), "spmv_resident": int(rng.choice([0, 1, 2]))}
        if rng.random() < 0.5:
            knobs["spmv_rows_per_wg"] = int(rng.integers(1, 64 * max(block, 64) // 64 + 1))
        else:
            knobs["spmv_wgs_per_cu"] = int(rng.choice([0, 1, 2, 3, 4]))
            knobs["spmv_steps_per_wave"] = int(rng.choice([0, 1, 3, 8, 40]))
        y = spmv_case(W, x, b_delta, **knobs)
        check_y(y, W, x, f"case {case}: {rows}x{cols} d={dens} b={b_delta} {knobs}")


RESIDENT_VARIANTS = {
    "auto": {},
    "never": {"spmv_resident": 1},
    "k1": {"spmv_resident": 2, "spmv_wgs_per_cu": 1},
    "k2_ring4": {"spmv_resident": 2, "spmv_wgs_per_cu": 2, "spmv_ring": 4},
    "k3_b320": {"spmv_resident": 2, "spmv_wgs_per_cu": 3, "spmv_block": 320},
    "k4": {"spmv_resident": 2, "spmv_wgs_per_cu": 4},
    "k1_b1024": {"spmv_resident": 2, "spmv_wgs_per_cu": 1, "spmv_block": 1024},
    "k2_b704": {"spmv_resident": 2, "spmv_wgs_per_cu": 2, "spmv_block": 704},
    "many_wgs_r40_b256": {"spmv_resident": 1, "spmv_rows_per_wg": 40, "spmv_block": 256},
    "many_wgs_r63_b64": {"spmv_resident": 1, "spmv_rows_per_wg": 63, "spmv_block": 64},
    "many_wgs_steps3": {"spmv_resident_steps": 1, "spmv_steps_per_wave": 3},
    "many_wgs_steps40": {"spmv_resident_steps": 1, "spmv_steps_per_wave": 40, "spmv_block": 192},
}


@pytest.mark.parametrize("variant", list(RESIDENT_VARIANTS))
def test_spmv_resident_round_launch_shapes(variant):
    """One resident round of workgroups (a multiple of the compute-unit count) with row counts
    that do not divide evenly: every row must still be computed exactly once, single and grouped."""
    W = wl.bernoulli(2311, 1536, 0.5, 0.02, 41, 1)
    W[100:140] = 0                                        # a run of empty rows inside one workgroup's share
    x = wl.x_vector(1536, 41, 1)
    y = spmv_case(W, x, spmv_kernel=2, **RESIDENT_VARIANTS[variant])
    check_y(y, W, x, variant)
    # grouped: three matrices of different heights and widths share the round
    specs = [(1500, 2048, 0.5), (1031, 1024, 0.6), (777, 4096, 0.4)]
    Ws = [wl.bernoulli(r, c, d, 0.02, 42, i) for i, (r, c, d) in enumerate(specs)]
    xs = [wl.x_vector(c, 42, i) for i, (_, c, _) in enumerate(specs)]
    for k, v in dict(spmv_kernel=2, **RESIDENT_VARIANTS[variant]).items():
        M.set_tuning(k, v)
    try:
        ms = [M.encode(Wi).to_device() for Wi in Ws]
        ys = M.spmv_group(ms, [to_dev(xi) for xi in xs])
        torch.cuda.synchronize()
    finally:
        for k in dict(spmv_kernel=2, **RESIDENT_VARIANTS[variant]):
            M.set_tuning(k, 0)
    for i, (Wi, xi, yi) in enumerate(zip(Ws, xs, ys)):
        check_y(yi, Wi, xi, f"{variant} group member {i}")


def test_spmv_under_graph_capture_and_on_two_streams():
    """The products only enqueue kernels, so they can be captured into a HIP graph and replayed,
    and one handle can be used from two streams at once."""
    W = wl.half_row_matrix(1024, 4096, 77)
    x1, x2 = wl.x_vector(4096, 43, 1), wl.x_vector(4096, 43, 2)
    m = M.encode(W).to_device()
    xd = to_dev(x1)
    y = torch.empty(1024, dtype=torch.float16, device="cuda")
    eager1 = m.spmv(to_dev(x1)).clone()
    eager2 = m.spmv(to_dev(x2)).clone()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        m.spmv(xd, y, stream=side)                       # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            m.spmv(xd, y, stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    for rep, (xv, want) in enumerate([(x1, eager1), (x2, eager2), (x1, eager1), (x2, eager2)]):
        xd.copy_(to_dev(xv))
        y.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, want), f"replay {rep}"
    # two streams, same handle, different vectors
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    xa, xb = to_dev(x1), to_dev(x2)
    ya = torch.empty(1024, dtype=torch.float16, device="cuda")
    yb = torch.empty(1024, dtype=torch.float16, device="cuda")
    torch.cuda.synchronize()
    for _ in range(20):
        m.spmv(xa, ya, stream=s1)
        m.spmv(xb, yb, stream=s2)
    torch.cuda.synchronize()
    assert torch.equal(ya, eager1) and torch.equal(yb, eager2)


def test_spmv_all_zero_matrix_and_zero_sized():
    x = wl.x_vector(640, 3, 3)
    y = spmv_case(np.zeros((77, 640), dtype=np.uint16), x, spmv_kernel=2)
    assert (y == 0).all()
    y = spmv_case(np.zeros((77, 640), dtype=np.uint16), x)
    assert (y == 0).all()
    m = M.encode(np.zeros((0, 640), dtype=np.uint16)).to_device()
    m.spmv(to_dev(x), torch.empty(0, dtype=torch.float16, device="cuda"))
    torch.cuda.synchronize()


def test_subnormal_weights_are_not_flushed():
    # every weight is an fp16 subnormal; x = 2048 makes the exact row sums O(1)
    rng = np.random.default_rng(1)
    R, C = 64, 2048
    W = np.zeros((R, C), dtype=np.uint16)
    mask = rng.random((R, C)) < 0.5
    W[mask] = rng.integers(1, 0x400, size=int(mask.sum()), dtype=np.uint16)   # positive subnormals
    x = np.full(C, np.float16(2048.0)).view(np.uint16)
    for variant in ("wave_row", "sub64"):
        y = spmv_case(W, x, **VARIANTS[variant])
        check_y(y, W, x, variant)
        y64, _ = oracle.dense_matvec(W, x)
        assert y64.min() > 10.0                                   # flushing would give exactly 0
        assert np.allclose(y.float().cpu().numpy(), y64, rtol=2e-3)


def test_unaligned_x_and_y_pointers():
    W = wl.bernoulli(150, 1000, 0.5, 0.02, 4, 4)
    x = wl.x_vector(1000, 4, 4)
    xbuf = torch.zeros(1001, dtype=torch.float16, device="cuda")
    xbuf[1:] = to_dev(x)
    ybuf = torch.zeros(151, dtype=torch.float16, device="cuda")
    m = M.encode(W).to_device()
    for kernel in (1, 2):
        M.set_tuning("spmv_kernel", kernel)
        m.spmv(xbuf[1:], ybuf[1:])
        torch.cuda.synchronize()
        check_y(ybuf[1:], W, x, f"kernel {kernel}")
    M.set_tuning("spmv_kernel", 0)


def test_x_larger_than_64k_lds_and_x_larger_than_lds():
    # 40000 columns need ~82 KB of LDS (above the 64 KB default limit)
    W = wl.bernoulli(40, 40000, 0.3, 0.02, 6, 1)
    x = wl.x_vector(40000, 6, 1)
    check_y(spmv_case(W, x, spmv_kernel=2), W, x, "80KB LDS wave_row")
    check_y(spmv_case(W, x, spmv_kernel=1, spmv_lanes=64), W, x, "80KB LDS sub64")
    # 100000 columns do not fit in LDS at all: x is gathered from global memory
    W = wl.bernoulli(24, 100000, 0.2, 0.02, 6, 2)
    x = wl.x_vector(100000, 6, 2)
    check_y(spmv_case(W, x), W, x, "global x")


def test_wrap_device_reuses_an_existing_encoding():
    W = wl.bernoulli(300, 2048, 0.5, 0.02, 8, 8)
    x = wl.x_vector(2048, 8, 8)
    m = M.encode(W).to_device()
    v, d, r = [b.clone() for b in m.device_buffers()]
    w = M.wrap_device(300, 2048, m.report.pad_nnz, v, d, r)
    y = w.spmv(to_dev(x))
    torch.cuda.synchronize()
    check_y(y, W, x, "wrapped")
    assert torch.equal(y, m.spmv(to_dev(x)))


# ------------------------------------------------------------------ other code widths

WIDTH_CASES = {
    "half_1200x3000": lambda: (wl.bernoulli(1200, 3000, 0.5, 0.02, 51, 1), wl.x_vector(3000, 51, 1)),
    "dense_300x1031": lambda: (wl.bernoulli(300, 1031, 1.0, 0.02, 51, 2), wl.x_vector(1031, 51, 2)),
    "sparse97_600x9000": lambda: (wl.bernoulli(600, 9000, 0.03, 1.0, 51, 3), wl.x_vector(9000, 51, 3)),
    "ragged_301x777": lambda: (wl.bernoulli(301, 777, 0.7, 0.02, 51, 4), wl.x_vector(777, 51, 4)),
    "c4_512x4096": lambda: (wl.config4(rows=512, cols=4096).W, wl.config4(rows=512, cols=4096).x),
    "one_row_20000": lambda: (wl.bernoulli(1, 20000, 0.3, 0.02, 51, 5), wl.x_vector(20000, 51, 5)),
}


@pytest.mark.parametrize("variant", ["auto", "sub32", "wave_row", "wave_row_b64_r200", "wave_row_b256_r37",
                                     "wave_row_align64", "wave_row_align256_b256_r37", "wave_row_align512"])
@pytest.mark.parametrize("b_delta", [1, 2, 8])
@pytest.mark.parametrize("case", list(WIDTH_CASES))
def test_spmv_other_code_widths(case, b_delta, variant):
    """1-, 2- and 8-bit codes: same product, same tolerance, on both kernels."""
    W, x = WIDTH_CASES[case]()
    y = spmv_case(W, x, b_delta, **VARIANTS[variant])
    check_y(y, W, x, f"{case}/b{b_delta}/{variant}")


@pytest.mark.parametrize("b_delta", [1, 2, 8])
def test_other_code_widths_gpu_encoder_wrap_and_groups(b_delta):
    W = wl.bernoulli(700, 2500, 0.35, 0.02, 52, b_delta)
    W[13] = 0
    x = wl.x_vector(2500, 52, 1)
    enc = oracle.encode(W, b_delta)
    g = M.encode_device(to_dev(W), b_delta=b_delta)
    assert_same_encoding(g.fetch_device(), enc)
    rep = g.get_report()
    assert (rep.nnz, rep.pad_nnz, rep.alloc_nnz, rep.b_delta) == (enc.nnz, enc.pad_nnz, enc.alloc_nnz, b_delta)
    check_y(g.spmv(to_dev(x)), W, x, f"device-encoded b{b_delta}")
    # adopt the same device arrays through the wrap call
    bufs = [torch.from_numpy(a.copy()).cuda() for a in g.fetch_device()]
    w = M.wrap_device(700, 2500, enc.pad_nnz, *bufs, b_delta=b_delta)
    assert torch.equal(w.spmv(to_dev(x)), g.spmv(to_dev(x)))
    # a group that mixes code widths: one launch per width, same results
    others = [M.encode(W, b).to_device() for b in (4, 2, 8)]
    ys = M.spmv_group([g] + others, [to_dev(x)] * 4)
    torch.cuda.synchronize()
    for i, yi in enumerate(ys):
        check_y(yi, W, x, f"mixed group member {i}")
    # the small-batch product decodes the same widths (1-bit codes: one vector at a time)
    X = torch.stack([to_dev(wl.x_vector(2500, 52, 10 + b)) for b in range(7)])
    Y = g.spmm(X)
    torch.cuda.synchronize()
    for b in range(7):
        check_y(Y[b], W, wl.x_vector(2500, 52, 10 + b), f"spmm b{b_delta} column {b}")


def test_code_widths_full_size_llama_shape():
    """4096 x 11008 at 50 % (2-bit codes) and at 97 % (8-bit codes), in the launch shape bench.py times."""
    for b_delta, density, stream in ((2, 0.5, 61), (8, 0.03, 62), (2, 0.75, 63)):
        W = wl.bernoulli(4096, 11008, density, 0.02, 53, stream)
        x = wl.x_vector(11008, 53, stream)
        m = M.encode(W, b_delta).to_device()
        check_y(m.spmv(to_dev(x)), W, x, f"b{b_delta} d{density}")


# ------------------------------------------------------------------ grouped launches

def test_spmv_group_mixed_shapes_one_call():
    specs = [(300, 2048, 0.5), (64, 4096, 0.5), (500, 1000, 0.3), (40, 8000, 0.9),   # wave-per-row kernel
             (200, 300, 0.5),                                                         # short rows: own launch
             (77, 640, 0.0),                                                          # nothing stored
             (10, 100000, 0.2),                                                       # x larger than LDS
             (129, 5000, 1.0)]
    Ws = [wl.bernoulli(r, c, d, 0.02, 31, i) if d > 0 else np.zeros((r, c), dtype=np.uint16)
          for i, (r, c, d) in enumerate(specs)]
    xs = [wl.x_vector(c, 31, i) for i, (_, c, _) in enumerate(specs)]
    ms = [M.encode(W).to_device() for W in Ws]
    xd = [to_dev(x) for x in xs]
    ys = M.spmv_group(ms, xd)
    torch.cuda.synchronize()
    for i, (W, x, y) in enumerate(zip(Ws, xs, ys)):
        check_y(y, W, x, f"group member {i} {specs[i]}")
    # the single-product call gives bit-identical results (same kernel, same order of operations)
    for m, x, y in zip(ms, xd, ys):
        assert torch.equal(m.spmv(x), y)
    # q/k/v style: three matrices, one shared x
    q = [M.encode(wl.half_row_matrix(256, 4096, 60 + i)).to_device() for i in range(3)]
    xq = to_dev(wl.x_vector(4096, 31, 99))
    yq = M.spmv_group(q, [xq, xq, xq])
    torch.cuda.synchronize()
    for i in range(3):
        check_y(yq[i], wl.half_row_matrix(256, 4096, 60 + i), wl.x_vector(4096, 31, 99), f"qkv {i}")


def test_group_argument_errors():
    lib = M.load_library()
    m = M.encode(wl.config1().W).to_device()
    x = to_dev(wl.config1().x)
    y = torch.empty(512, dtype=torch.float16, device="cuda")
    import ctypes
    VP = ctypes.c_void_p * 9
    hs = VP(*[m._h.value] * 9); xs = VP(*[x.data_ptr()] * 9); ys = VP(*[y.data_ptr()] * 9)
    assert lib.macko_spmv_group(0, hs, xs, ys, None) == -1
    assert lib.macko_spmv_group(9, hs, xs, ys, None) == -1
    unbound = M.encode(wl.config1().W)
    hs2 = VP(*([m._h.value] * 8 + [unbound._h.value]))
    hs2[1] = unbound._h.value
    assert lib.macko_spmv_group(2, hs2, xs, ys, None) == -5
    torch.cuda.synchronize()


def test_dense_gemv_group():
    shapes = [(300, 1024), (64, 4096), (33, 777), (128, 8200)]
    Ws = [wl.bernoulli(r, c, 1.0, 0.02, 41, i) for i, (r, c) in enumerate(shapes)]
    xs = [wl.x_vector(c, 41, i) for i, (_, c) in enumerate(shapes)]
    ys = M.dense_gemv_group([to_dev(W) for W in Ws], [to_dev(x) for x in xs])
    torch.cuda.synchronize()
    for W, x, y, shp in zip(Ws, xs, ys, shapes):
        check_y(y, W, x, f"gemv group {shp}")


# ------------------------------------------------------------------ small-batch products

def check_Y(Y_dev, W, X, what):
    for b in range(X.shape[0]):
        check_y(Y_dev[b], W, X[b], f"{what} vector {b}")


@pytest.mark.parametrize("batch", [1, 2, 3, 4, 5, 7, 8, 11, 16])
def test_spmm_batches(batch):
    W = wl.bernoulli(333, 2000, 0.5, 0.02, 51, 1)
    W[5] = 0
    W[100:110] = 0
    X = np.stack([wl.x_vector(2000, 51, 10 + b) for b in range(batch)])
    m = M.encode(W).to_device()
    Y = m.spmm(to_dev(X))
    torch.cuda.synchronize()
    assert Y.shape == (batch, 333)
    check_Y(Y, W, X, f"batch {batch}")
    assert (Y[:, 5] == 0).all() and (Y[:, 100:110] == 0).all()
    # each vector agrees with the matrix-vector kernel to within both tolerances
    y0 = m.spmv(to_dev(X[0]))
    assert torch.allclose(Y[0].float(), y0.float(), atol=2e-3, rtol=2e-2)


def test_spmm_shapes_strides_and_fallbacks():
    cases = [
        (wl.bernoulli(70, 5000, 0.6, 0.02, 52, 1), 8),        # long rows
        (wl.bernoulli(40, 12000, 0.3, 0.02, 52, 2), 8),       # 8 vectors do not fit LDS: pieces of 4
        (wl.bernoulli(24, 30000, 0.2, 0.02, 52, 3), 6),       # pieces of 2
        (wl.bernoulli(10, 100000, 0.2, 0.02, 52, 4), 3),      # x larger than LDS: vector by vector
        (wl.bernoulli(200, 300, 0.5, 0.02, 52, 5), 4),        # short rows: vector by vector
        (wl.config4(rows=128, cols=2048).W, 8),
        (np.zeros((50, 640), dtype=np.uint16), 5),
        (wl.bernoulli(129, 1001, 1.0, 0.02, 52, 6), 8),       # dense, odd column count
    ]
    for i, (W, batch) in enumerate(cases):
        C = W.shape[1]
        X = np.stack([wl.x_vector(C, 52, 100 * i + b) for b in range(batch)])
        m = M.encode(W).to_device()
        # strided, unaligned X and Y
        Xbuf = torch.zeros((batch, C + 9), dtype=torch.float16, device="cuda")
        Xbuf[:, 1:C + 1] = to_dev(X)
        Ybuf = torch.full((batch, W.shape[0] + 5), 7.0, dtype=torch.float16, device="cuda")
        m.spmm(Xbuf[:, 1:C + 1], Ybuf[:, 3:3 + W.shape[0]])
        torch.cuda.synchronize()
        check_Y(Ybuf[:, 3:3 + W.shape[0]], W, X, f"case {i}")
        assert (Ybuf[:, :3] == 7).all() and (Ybuf[:, 3 + W.shape[0]:] == 7).all()


@pytest.mark.parametrize("batch", [2, 4, 8, 13])
@pytest.mark.parametrize("kind", ["b1", "b2", "b4", "b8", "fp8"])
def test_spmm_batch_kernel_every_code_width_and_8_bit_values(kind, batch):
    """The batch kernel proper (rows long enough for it): one decode per stored entry, `batch` products.
    Row lengths straddle steps, rows start inside chunks, some rows are empty."""
    b_delta = {"b1": 1, "b2": 2, "b4": 4, "b8": 8, "fp8": 4}[kind]
    density = {"b1": 0.9, "b2": 0.6, "b4": 0.5, "b8": 0.25, "fp8": 0.5}[kind]
    rows, cols = 150, 4100
    W = wl.bernoulli(rows, cols, density, 0.02, 54, b_delta)
    W[7] = 0
    W[40:43] = 0
    X = np.stack([wl.x_vector(cols, 54, 10 * batch + b) for b in range(batch)])
    if kind == "fp8":
        W8 = wl.fp8_values_of(W)
        m = M.encode_fp8(W8).to_device()
        assert m.report.pad_nnz // rows >= 384
        Y = m.spmm(to_dev(X))
        torch.cuda.synchronize()
        for b in range(batch):
            check_y8(Y[b], W8, X[b], f"fp8 batch {batch} vector {b}")
        y0 = m.spmv(to_dev(X[0]))
    else:
        m = M.encode(W, b_delta).to_device()
        assert m.report.pad_nnz // rows >= 384
        Y = m.spmm(to_dev(X))
        torch.cuda.synchronize()
        check_Y(Y, W, X, f"{kind} batch {batch}")
        y0 = m.spmv(to_dev(X[0]))
    torch.cuda.synchronize()
    assert (Y[:, 7] == 0).all() and (Y[:, 40:43] == 0).all()
    assert torch.allclose(Y[0].float(), y0.float(), atol=2e-3, rtol=2e-2)


def test_spmm_llama_shape_full_size():
    case = next(iter(wl.config2()))
    X = np.stack([wl.x_vector(case.cols, 53, b) for b in range(8)])
    m = M.encode(case.W).to_device()
    Y = m.spmm(to_dev(X))
    torch.cuda.synchronize()
    check_Y(Y, case.W, X, case.name)


# ------------------------------------------------------------------ GPU encoder

ENC_CASES = {
    "c1": lambda: wl.config1().W,
    "ragged": lambda: wl.bernoulli(301, 777, 0.5, 0.02, 9, 1),
    "very_sparse": lambda: wl.bernoulli(200, 3000, 0.02, 1.0, 9, 3),
    "dense": lambda: wl.bernoulli(100, 1031, 1.0, 0.02, 9, 4),
    "c4": lambda: wl.config4(rows=256, cols=2048).W,
    "c4b": lambda: wl.config4b(rows=128, cols=2048).W,
    "one_col": lambda: wl.bernoulli(300, 1, 0.5, 1.0, 9, 6),
    "empty": lambda: np.zeros((50, 600), dtype=np.uint16),
    "llama_slice": lambda: wl.half_row_matrix(512, 4096, 42),
}


@pytest.mark.parametrize("case", list(ENC_CASES))
def test_gpu_encoder_is_bit_exact(case):
    W = ENC_CASES[case]()
    enc = oracle.encode(W)
    g = M.encode_device(to_dev(W))
    assert_same_encoding(g.fetch_device(), enc)
    rep = g.report
    assert (rep.nnz, rep.pad_nnz, rep.alloc_nnz) == (enc.nnz, enc.pad_nnz, enc.alloc_nnz)
    ent = np.diff(enc.row_ptr.astype(np.int64))
    assert rep.empty_rows == int((ent == 0).sum()) and rep.max_row_entries == int(ent.max(initial=0))
    assert rep.total_bytes == enc.total_bytes
    # and the device-encoded handle multiplies correctly
    x = wl.x_vector(W.shape[1], 1, 1)
    y = g.spmv(to_dev(x))
    torch.cuda.synchronize()
    check_y(y, W, x, case)


def test_gpu_encoder_special_values_and_strided_unaligned_input():
    W = wl.bernoulli(64, 1001, 0.3, 0.02, 2, 2)
    W[0, 3] = 0x8000
    W[0, 5] = 0x0001
    W[1, 0] = 0x7C00
    W[2, 50] = 0xFE00
    W[5, 17] = 0x8001
    enc = oracle.encode(W)
    big = torch.zeros((64, 1003), dtype=torch.float16, device="cuda")     # ld = 1003: no 16-byte rows
    big[:, 1:1002] = to_dev(W)
    g = M.encode_device(big[:, 1:1002])
    assert_same_encoding(g.fetch_device(), enc)
    # the host encoder bound to the device gives the same bytes
    h = M.encode(W).to_device()
    assert_same_encoding(h.fetch_device(), enc)


# ------------------------------------------------------------------ dense GEMV baseline

@pytest.mark.parametrize("shape", [(512, 512), (300, 1000), (77, 4096), (64, 8200), (10, 40000), (33, 777), (5, 3)])
def test_dense_gemv(shape):
    R, C = shape
    W = wl.bernoulli(R, C, 1.0, 0.02, 12, R)
    x = wl.x_vector(C, 12, R)
    y = M.dense_gemv(to_dev(W), to_dev(x))
    torch.cuda.synchronize()
    check_y(y, W, x, f"gemv {shape}")
    for knobs in ({"gemv_block": 256, "gemv_rows_per_wg": 3}, {"gemv_block": 1024, "gemv_rows_per_wg": 1000}):
        for k, v in knobs.items():
            M.set_tuning(k, v)
        y = M.dense_gemv(to_dev(W), to_dev(x))
        torch.cuda.synchronize()
        check_y(y, W, x, f"gemv {shape} {knobs}")
        for k in knobs:
            M.set_tuning(k, 0)


def test_dense_gemv_with_leading_dimension_and_on_sparse_input():
    W = wl.half_row_matrix(200, 1024, 5)
    x = wl.x_vector(1024, 5, 5)
    big = torch.zeros((200, 1040), dtype=torch.float16, device="cuda")
    big[:, :1024] = to_dev(W)
    y = M.dense_gemv(big[:, :1024], to_dev(x))
    torch.cuda.synchronize()
    check_y(y, W, x, "ld=1040")
    # sparse and dense paths agree on the same matrix to within both tolerances
    ys = spmv_case(W, x)
    assert torch.allclose(ys.float(), y.float(), atol=2e-3, rtol=2e-2)


# ------------------------------------------------------------------ full-size configurations

def grouped_like_the_bench(handles, xs, singles):
    """The launches bench.py times: {q,k,v}, {o}, {gate,up}, {down}, and all seven at once.  Every product
    must come out exactly as from its own launch (the arithmetic per row does not depend on the launch shape)."""
    sq, gu, dn = handles
    xq, xg, xd = xs
    yq, yg, yd = singles
    for group, xv, want in (([sq] * 3, [xq] * 3, [yq] * 3), ([sq], [xq], [yq]), ([gu] * 2, [xg] * 2, [yg] * 2),
                            ([dn], [xd], [yd]),
                            ([sq] * 4 + [gu] * 2 + [dn], [xq] * 4 + [xg] * 2 + [xd], [yq] * 4 + [yg] * 2 + [yd])):
        got = M.spmv_group(group, xv)
        torch.cuda.synchronize()
        for g, w in zip(got, want):
            assert torch.equal(g, w)


def test_config2_llama2_7b_shapes_full_size():
    handles, xs, singles = [], [], []
    for case in wl.config2():
        enc = oracle.encode(case.W)
        m = M.encode(case.W)
        assert_same_encoding(m.host_buffers(), enc)
        m.to_device()
        y = m.spmv(to_dev(case.x))
        torch.cuda.synchronize()
        check_y(y, case.W, case.x, case.name)
        handles.append(m); xs.append(to_dev(case.x)); singles.append(y)
        yd = M.dense_gemv(to_dev(case.W), to_dev(case.x))
        torch.cuda.synchronize()
        check_y(yd, case.W, case.x, case.name + " dense")
        g = M.encode_device(to_dev(case.W))
        assert_same_encoding(g.fetch_device(), enc)
    grouped_like_the_bench(handles, xs, singles)


@pytest.mark.parametrize("sparsity", wl.SWEEP_SPARSITIES)
def test_config3_sweep_matrix_full_size(sparsity):
    """Every level of the sparsity sweep at its full size: both encoders byte for byte against the
    oracle's encoding, y against the dense product by definition."""
    case = wl.config3(sparsity)
    enc = oracle.encode(case.W)
    m = M.encode(case.W)
    assert_same_encoding(m.host_buffers(), enc)
    m.to_device()
    y = m.spmv(to_dev(case.x))
    torch.cuda.synchronize()
    check_y(y, case.W, case.x, case.name)
    rep = m.report
    assert rep.effd_best <= rep.effd + 1e-9
    assert rep.pad_nnz == enc.pad_nnz and rep.padding_entries == enc.pad_nnz - enc.nnz
    assert_same_encoding(m.fetch_device(), enc)
    g = M.encode_device(to_dev(case.W))
    assert_same_encoding(g.fetch_device(), enc)
    yg = g.spmv(to_dev(case.x))
    torch.cuda.synchronize()
    assert torch.equal(yg, y)


def test_config4_adversarial_full_size():
    for case in (wl.config4(), wl.config4b()):
        enc = oracle.encode(case.W)
        m = M.encode(case.W)
        assert_same_encoding(m.host_buffers(), enc)
        m.to_device()
        y = m.spmv(to_dev(case.x))
        torch.cuda.synchronize()
        check_y(y, case.W, case.x, case.name)
        g = M.encode_device(to_dev(case.W))
        assert_same_encoding(g.fetch_device(), enc)


def test_config5_llama2_13b_layer_shapes_full_size():
    handles, xs, singles = [], [], []
    for case in wl.config5_layer():
        m = M.encode(case.W).to_device()
        y = m.spmv(to_dev(case.x))
        torch.cuda.synchronize()
        check_y(y, case.W, case.x, case.name)
        handles.append(m); xs.append(to_dev(case.x)); singles.append(y)
    grouped_like_the_bench(handles, xs, singles)


def test_config5_whole_stack_as_the_bench_issues_it():
    """The 224 products of the 32-layer 13B-shaped stack, built the way bench.py builds them (one layer's
    three matrices, the device buffers replicated to 224 distinct addresses: the first copy from the host
    encoder, the others from the GPU encoder), once through macko_spmv_many and once as the 128 grouped
    launches {q,k,v}, {o}, {gate,up}, {down} per layer.  Every one of the 448 results is compared with the
    oracle's dense product of its matrix."""
    plan = [("qkvo", 4), ("gate_up", 2), ("down", 1)]
    handles, xs, want = {}, {}, {}
    for case, (tag, mult) in zip(wl.config5_layer(), plan):
        enc = oracle.encode(case.W)
        first = M.encode(case.W).to_device()
        Wd = to_dev(case.W)
        hs = [first] + [M.encode_device(Wd) for _ in range(32 * mult - 1)]
        del Wd
        assert_same_encoding(hs[-1].fetch_device(), enc)
        handles[tag], xs[tag] = hs, to_dev(case.x)
        y64, s64 = oracle.dense_matvec(case.W, case.x)
        want[tag] = (y64, REL_TOL * s64 + ABS_TOL)

    def check(tag, y, what):
        y64, bound = want[tag]
        got = y.float().cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all(), what
        assert (np.abs(got - y64) <= bound).all(), what

    seq = [(tag, layer * mult + k) for layer in range(32) for tag, mult in plan for k in range(mult)]
    assert len(seq) == 224
    # one library call
    ys = [torch.full((handles[t][0].rows,), float("nan"), dtype=torch.float16, device="cuda") for t, _ in seq]
    many = M.SpmvMany([handles[t][c] for t, c in seq], [xs[t] for t, _ in seq], ys)
    many.launch()
    torch.cuda.synchronize()
    for i, (t, c) in enumerate(seq):
        check(t, ys[i], f"spmv_many product {i} ({t} copy {c})")
    first_of = {t: next(ys[i] for i, (tt, _) in enumerate(seq) if tt == t) for t, _ in plan}
    for i, (t, _) in enumerate(seq):                      # same bytes, same kernel arithmetic: same bits
        assert torch.equal(ys[i], first_of[t])
    # 128 grouped launches on one stream
    n_launches = 0
    for layer in range(32):
        for tag, ks in (("qkvo", [0, 1, 2]), ("qkvo", [3]), ("gate_up", [0, 1]), ("down", [0])):
            mult = dict(plan)[tag]
            hs = [handles[tag][layer * mult + k] for k in ks]
            out = [torch.full((hs[0].rows,), float("nan"), dtype=torch.float16, device="cuda") for _ in ks]
            M.SpmvGroup(hs, [xs[tag]] * len(ks), out).launch()
            n_launches += 1
            torch.cuda.synchronize()
            for k, yk in zip(ks, out):
                check(tag, yk, f"grouped launch layer {layer} {tag}[{k}]")
    assert n_launches == 128


# Appendix D: the 31 matrix shapes of the paper's runtime sweep, each at its full size.
_APPD_SMALLEST = sorted(wl.APPENDIX_D_SHAPES, key=lambda rc: rc[0] * rc[1])[:5]
_APPD_CASES = [(r, c, 50) for r, c in wl.APPENDIX_D_SHAPES] + [(r, c, 90) for r, c in _APPD_SMALLEST]


@pytest.mark.parametrize("rows,cols,sparsity", _APPD_CASES, ids=[f"{r}x{c}_s{s}" for r, c, s in _APPD_CASES])
def test_appendix_d_shapes_full_size(rows, cols, sparsity):
    case = wl.appendix_d_case(rows, cols, sparsity)
    m = M.encode(case.W).to_device()
    y = m.spmv(to_dev(case.x))
    torch.cuda.synchronize()
    check_y(y, case.W, case.x, case.name)
    yd = M.dense_gemv(to_dev(case.W), to_dev(case.x))
    torch.cuda.synchronize()
    check_y(yd, case.W, case.x, case.name + " dense")


# ------------------------------------------------------------------ expanding the format on the device

EXPAND_CASES = dict(WIDTH_CASES)
EXPAND_CASES["empty_rows_257x1500"] = lambda: (_with_empty_rows(wl.bernoulli(257, 1500, 0.4, 0.02, 61, 1)),
                                                wl.x_vector(1500, 61, 1))
EXPAND_CASES["first_nonzero_late_64x5000"] = lambda: (_late_start(wl.bernoulli(64, 5000, 0.6, 0.02, 61, 2)),
                                                       wl.x_vector(5000, 61, 2))
# row buffers of the one-pass decoder: two wavefronts per workgroup, one, and rows too long for LDS
EXPAND_CASES["wide_6x30000"] = lambda: (wl.bernoulli(6, 30000, 0.5, 0.02, 61, 3), wl.x_vector(30000, 61, 3))
EXPAND_CASES["wide_5x45000"] = lambda: (wl.bernoulli(5, 45000, 0.4, 0.02, 61, 4), wl.x_vector(45000, 61, 4))
EXPAND_CASES["exactly_lds_2x81920"] = lambda: (wl.bernoulli(2, 81920, 0.2, 0.02, 61, 6), wl.x_vector(81920, 61, 6))
EXPAND_CASES["just_over_lds_2x81928"] = lambda: (wl.bernoulli(2, 81928, 0.2, 0.02, 61, 7), wl.x_vector(81928, 61, 7))
EXPAND_CASES["too_wide_for_lds_3x90000"] = lambda: (wl.bernoulli(3, 90000, 0.3, 0.02, 61, 5),
                                                     wl.x_vector(90000, 61, 5))


def _with_empty_rows(W):
    W[0] = 0
    W[100:131] = 0
    W[-1] = 0
    return W


def _late_start(W):
    W[:, :3000] = 0            # every row starts with padding entries only
    W[5, :] = 0
    W[5, 4999] = 0x3C00        # a row whose only non-zero is in the last column
    return W


@pytest.mark.parametrize("b_delta", [1, 2, 4, 8])
@pytest.mark.parametrize("case", list(EXPAND_CASES))
def test_columns_on_the_device_equal_the_oracles(case, b_delta):
    """Index reconstruction (Section 4.4, Alg. 1) in isolation: the column index of every stored
    entry, formed with the decode and the wavefront prefix sum the product uses, bit for bit."""
    W, _ = EXPAND_CASES[case]()
    enc = oracle.encode(W, b_delta)
    _, want = oracle.unpack(enc)
    m = M.encode(W, b_delta).to_device()
    got = m.columns_device()
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    assert got.shape[0] == max(enc.alloc_nnz, 1)
    assert np.array_equal(got[: enc.pad_nnz], want)
    assert (got[enc.pad_nnz:] == -1).all()                 # the tail is not touched


@pytest.mark.parametrize("b_delta", [1, 2, 4, 8])
@pytest.mark.parametrize("case", list(EXPAND_CASES))
def test_decode_on_the_device_round_trips_exactly(case, b_delta):
    W, _ = EXPAND_CASES[case]()
    want = oracle.decode(oracle.encode(W, b_delta))
    m = M.encode_device(to_dev(W), b_delta=b_delta)       # device encoder -> device decoder
    back = m.decode_device()
    torch.cuda.synchronize()
    assert np.array_equal(back.cpu().numpy().view(np.uint16), want)
    # into a wider, unaligned buffer: cells beyond cols keep their contents
    rows, cols = W.shape
    buf = torch.full((rows, cols + 5), 7.0, dtype=torch.float16, device="cuda")
    view = buf[:, 1: 1 + cols]
    rc = M.load_library().macko_decode_device(m._h, view.data_ptr(), buf.stride(0), 0)
    assert rc == 0
    torch.cuda.synchronize()
    host = buf.cpu().numpy().view(np.uint16)
    assert np.array_equal(host[:, 1: 1 + cols], want)
    assert (host[:, 0] == 0x4700).all() and (host[:, 1 + cols:] == 0x4700).all()


def test_expand_special_values_errors_and_full_size():
    W = wl.bernoulli(130, 900, 0.5, 0.02, 62, 1)
    W[3, 10:20] = [0x7C00, 0xFC00, 0x7E00, 0x0001, 0x8001, 0x8000, 0x0000, 0x7BFF, 0xFBFF, 0x03FF]
    m = M.encode(W).to_device()
    back = m.decode_device()
    torch.cuda.synchronize()
    assert np.array_equal(back.cpu().numpy().view(np.uint16), oracle.decode(oracle.encode(W)))
    lib = M.load_library()
    unbound = M.encode(W)
    rc = lib.macko_decode_device(unbound._h, back.data_ptr(), 900, 0)
    assert rc < 0 and "no device buffers" in M.status_string(rc)
    assert lib.macko_decode_device(m._h, back.data_ptr(), 899, 0) < 0          # ld < cols
    assert lib.macko_decode_device(m._h, 0, 900, 0) < 0
    assert lib.macko_columns_device(m._h, 0, 0) < 0
    assert lib.macko_columns_device(unbound._h, back.data_ptr(), 0) < 0
    # all-zero and zero-sized matrices
    z = M.encode(np.zeros((5, 64), dtype=np.uint16)).to_device()
    out = torch.full((5, 64), 3.0, dtype=torch.float16, device="cuda")
    z.decode_device(out)
    torch.cuda.synchronize()
    assert (out == 0).all()
    assert (z.columns_device().cpu().numpy() == -1).all()
    # one decoder-layer shape at full size, both ways
    case = list(wl.config2())[1]
    enc = oracle.encode(case.W)
    g = M.encode_device(to_dev(case.W))
    cols = g.columns_device()
    dense = g.decode_device()
    torch.cuda.synchronize()
    assert np.array_equal(cols.cpu().numpy()[: enc.pad_nnz], oracle.unpack(enc)[1])
    assert np.array_equal(dense.cpu().numpy().view(np.uint16), oracle.decode(enc))


# ------------------------------------------------------------------ checking adopted device arrays

@pytest.mark.parametrize("b_delta", [1, 2, 4, 8])
def test_check_device_accepts_valid_encodings_and_names_the_first_bad_row(b_delta):
    """Mistakes are planted in host copies of a valid encoding (made by the oracle), the copies are
    adopted with macko_wrap_device, and macko_check_device must name the first row that is wrong.
    No planted mistake makes a kernel read outside the arrays: bad pointers are reported undecoded."""
    rows, cols = 300, 2100
    W = wl.bernoulli(rows, cols, 0.4, 0.02, 71, b_delta)
    W[17] = 0
    W[299, cols - 1] = 0x3C00                                  # the last row reaches the last column
    enc = oracle.encode(W, b_delta)

    def wrapped(values, deltas, row_ptr, pad_nnz=None, ncols=cols):
        v = torch.from_numpy(values.copy()).cuda()
        d = torch.from_numpy(deltas.copy()).cuda()
        r = torch.from_numpy(row_ptr.astype(np.int64).astype(np.uint32).view(np.int32).copy()).cuda()
        return M.wrap_device(rows, ncols, enc.pad_nnz if pad_nnz is None else pad_nnz, v, d, r, b_delta)

    assert wrapped(enc.values, enc.deltas, enc.row_ptr).check_device() is None
    assert M.encode(W, b_delta).to_device().check_device() is None
    assert M.encode_device(to_dev(W), b_delta=b_delta).check_device() is None

    # one column too few: exactly the rows that reach the last column are wrong (row 299 does; find the first)
    _, colidx = oracle.unpack(enc)
    reach = [r for r in range(rows) if enc.row_ptr[r + 1] > enc.row_ptr[r] and colidx[enc.row_ptr[r + 1] - 1] == cols - 1]
    assert wrapped(enc.values, enc.deltas, enc.row_ptr, ncols=cols - 1).check_device() == reach[0]

    rp = enc.row_ptr.astype(np.int64)
    bad = rp.copy(); bad[0] = 8
    assert wrapped(enc.values, enc.deltas, bad).check_device() == 0                 # does not start at 0
    assert rp[119] > 0
    bad = rp.copy(); bad[120] = rp[119] - 1
    assert wrapped(enc.values, enc.deltas, bad).check_device() == 119              # decreasing
    bad = rp.copy(); bad[200] = enc.pad_nnz + 4096
    assert wrapped(enc.values, enc.deltas, bad).check_device() == 199              # beyond the arrays
    bad = rp.copy(); bad[rows] = enc.pad_nnz - 1
    assert wrapped(enc.values, enc.deltas, bad, pad_nnz=enc.pad_nnz).check_device() == rows - 1   # does not end at pad_nnz
    # a row boundary moved forward by a few entries: the row above it now decodes entries of the next row
    # and, being long enough, runs past the last column
    bad = rp.copy(); bad[51] = rp[53]
    got = wrapped(enc.values, enc.deltas, bad).check_device()
    assert got in (50, 51, 52)
    # all-zero and empty
    z = M.encode(np.zeros((4, 16), dtype=np.uint16), b_delta).to_device()
    assert z.check_device() is None
    lib = M.load_library()
    assert lib.macko_check_device(M.encode(W, b_delta)._h, 0, None) < 0             # not bound


# ------------------------------------------------------------------ 8-bit values

def check_y8(y_dev, W8, x, what=""):
    y64, s64 = oracle.dense_matvec8(W8, x)
    y = y_dev.float().cpu().numpy().astype(np.float64)
    err = np.abs(y - y64)
    tol = 1e-2 * s64 + 1e-3
    assert (err <= tol).all(), f"{what}: worst excess {float((err - tol).max()):.3e} at row {int((err - tol).argmax())}"


def test_fp8_every_bit_pattern_is_converted_like_the_oracle():
    """One row per E4M3 pattern (NaNs aside), a single entry each, x = 1: y must be the value itself,
    exactly (every E4M3 number is an fp16 number), including subnormals and both signs."""
    codes = np.array([c for c in range(256) if (c & 0x7F) not in (0, 0x7F)], dtype=np.uint8)
    W = np.zeros((len(codes), 512), dtype=np.uint8)
    W[np.arange(len(codes)), (np.arange(len(codes)) * 37) % 512] = codes
    W = np.repeat(W, 3, axis=0)                         # several rows per wavefront
    x = np.full(512, 0x3C00, dtype=np.uint16)
    m = M.encode_fp8(W).to_device()
    y = m.spmv(to_dev(x))
    torch.cuda.synchronize()
    want = oracle.fp8_to_double(np.repeat(codes, 3))
    assert np.array_equal(y.float().cpu().numpy().astype(np.float64), want)


FP8_CASES = {
    "half_1200x3000": lambda: wl.fp8_case(1200, 3000, 50),
    "dense_300x1031": lambda: wl.fp8_case(300, 1031, 0),
    "sparse90_600x9000": lambda: wl.fp8_case(600, 9000, 90),
    "ragged_301x777": lambda: wl.fp8_case(301, 777, 30),
    "one_row_20000": lambda: wl.fp8_case(1, 20000, 70),
    "short_rows_2000x96": lambda: wl.fp8_case(2000, 96, 50),
}


@pytest.mark.parametrize("variant", ["auto", "resident", "many_wgs_b256", "many_wgs_r37_b128", "align64",
                                     "align512_b256"])
@pytest.mark.parametrize("case", list(FP8_CASES))
def test_spmv_with_8_bit_values(case, variant):
    knobs = {"auto": {}, "resident": {"spmv_resident": 2}, "many_wgs_b256": {"spmv_resident": 1, "spmv_block": 256},
             "many_wgs_r37_b128": {"spmv_resident": 1, "spmv_rows_per_wg": 37, "spmv_block": 128},
             "align64": {"spmv_step_align": 64}, "align512_b256": {"spmv_step_align": 512, "spmv_block": 256}}[variant]
    c = FP8_CASES[case]()
    W = c.W.copy()
    if W.shape[0] > 40:
        W[10:30] = 0                                    # a run of empty rows
    enc = oracle.encode8(W, 4)
    for k, v in knobs.items():
        M.set_tuning(k, v)
    try:
        m = M.encode_fp8(W).to_device()
        v, d, r = m.fetch_device()
        assert np.array_equal(v, enc.values) and np.array_equal(d, enc.deltas) and np.array_equal(r, enc.row_ptr)
        y = m.spmv(to_dev(c.x))
        torch.cuda.synchronize()
    finally:
        for k in knobs:
            M.set_tuning(k, 0)
    check_y8(y, W, c.x, f"{case}/{variant}")
    if W.shape[0] > 40:
        assert (y[10:30] == 0).all()
    g = M.encode_device_fp8(torch.from_numpy(W).cuda())        # the GPU encoder: same bytes, same report
    gv, gd, gr = g.fetch_device()
    assert np.array_equal(gv, enc.values) and np.array_equal(gd, enc.deltas) and np.array_equal(gr, enc.row_ptr)
    rep = g.get_report()
    assert (rep.b_val, rep.nnz, rep.pad_nnz, rep.alloc_nnz, rep.total_bytes) == \
        (8, enc.nnz, enc.pad_nnz, enc.alloc_nnz, enc.total_bytes)
    for k, v in knobs.items():                          # same launch shape, hence the same summation order
        M.set_tuning(k, v)
    try:
        yg = g.spmv(to_dev(c.x))
    finally:
        for k in knobs:
            M.set_tuning(k, 0)
    assert torch.equal(yg, y)
    assert m.check_device() is None
    assert np.array_equal(m.columns_device().cpu().numpy()[: enc.pad_nnz], oracle.unpack(enc)[1])


def test_fp8_groups_unsupported_calls_and_full_size():
    lib = M.load_library()
    a, b = wl.fp8_case(700, 2048, 50), wl.fp8_case(900, 1024, 60)
    c16 = wl.appendix_d_case(500, 2048, 50)
    ma, mb, mc = M.encode_fp8(a.W).to_device(), M.encode_fp8(b.W).to_device(), M.encode(c16.W).to_device()
    ys = M.spmv_group([ma, mc, mb], [to_dev(a.x), to_dev(c16.x), to_dev(b.x)])      # mixed value widths, one call
    torch.cuda.synchronize()
    check_y8(ys[0], a.W, a.x, "group/a")
    check_y(ys[1], c16.W, c16.x, "group/16-bit")
    check_y8(ys[2], b.W, b.x, "group/b")
    # adopt a copy of the device arrays (a checkpoint loaded elsewhere)
    v, d, r = [t.clone() for t in ma.device_buffers()]
    w = M.wrap_device_fp8(700, 2048, ma.report.pad_nnz, v, d, r)
    assert w.get_report().b_val == 8 and w.check_device() is None
    yw = w.spmv(to_dev(a.x))
    torch.cuda.synchronize()
    assert torch.equal(yw, ys[0])
    # a batch of vectors: the batch kernel, a piece of 8 and a piece of 4 (3 used)
    xs = [wl.x_vector(2048, 88, i) for i in range(11)]
    X = torch.stack([to_dev(v) for v in xs])
    Y = ma.spmm(X)
    torch.cuda.synchronize()
    assert Y.shape == (11, 700)
    for i in (0, 7, 8, 10):
        check_y8(Y[i], a.W, xs[i], f"spmm/vector {i}")
    # the dense matrix back on the device, as bytes: aligned, and into a wider unaligned buffer
    for m, c in ((ma, a), (mb, b)):
        want = oracle.decode8(oracle.encode8(c.W, 4))
        back = m.decode_device()
        torch.cuda.synchronize()
        assert back.dtype == torch.uint8 and np.array_equal(back.cpu().numpy(), want)
        rows, cols = c.W.shape
        buf = torch.full((rows, cols + 5), 0x77, dtype=torch.uint8, device="cuda")
        assert lib.macko_decode_device(m._h, buf[:, 3:].data_ptr(), buf.stride(0), 0) == 0
        torch.cuda.synchronize()
        host = buf.cpu().numpy()
        assert np.array_equal(host[:, 3: 3 + cols], want)
        assert (host[:, :3] == 0x77).all() and (host[:, 3 + cols:] == 0x77).all()
    # the layer shapes at full size
    for (r, c) in ((4096, 4096), (11008, 4096), (4096, 11008)):
        case = wl.fp8_case(r, c, 50)
        m = M.encode_fp8(case.W).to_device()
        y = m.spmv(to_dev(case.x))
        torch.cuda.synchronize()
        check_y8(y, case.W, case.x, case.name)


def test_fp8_gpu_encoder_special_patterns_and_strided_unaligned_input():
    rng = np.random.default_rng(81)
    W = rng.integers(0, 256, size=(123, 1001), dtype=np.uint8)
    W[rng.random(W.shape) < 0.6] = 0
    W[3, 10:16] = [0x80, 0x7F, 0xFF, 0x01, 0x81, 0x00]      # -0 is a zero; NaN patterns and subnormals are values
    W[7] = 0
    enc = oracle.encode8(W, 4)
    big = torch.zeros((123, 1001 + 11), dtype=torch.uint8, device="cuda")
    big[:, 3: 3 + 1001] = torch.from_numpy(W).cuda()
    view = big[:, 3: 3 + 1001]                               # unaligned start, odd leading dimension
    lib = M.load_library()
    import ctypes
    h = ctypes.c_void_p()
    assert lib.macko_encode_device_fp8(view.data_ptr(), 123, 1001, big.stride(0), 0, ctypes.byref(h), None) == 0
    g = M.binding.MackoMatrix(h.value, None)
    gv, gd, gr = g.fetch_device()
    assert np.array_equal(gv, enc.values) and np.array_equal(gd, enc.deltas) and np.array_equal(gr, enc.row_ptr)
    # a layer shape at full size, against the host encoder's bytes
    case = wl.fp8_case(11008, 4096, 50)
    hv, hd, hr = M.encode_fp8(case.W).host_buffers()
    gv, gd, gr = M.encode_device_fp8(torch.from_numpy(case.W).cuda()).fetch_device()
    assert np.array_equal(gv, hv) and np.array_equal(gd, hd) and np.array_equal(gr, hr)
    assert np.array_equal(hv, oracle.encode8(case.W, 4).values)


# ------------------------------------------------------------------ maximum sizes

def test_more_than_2_pow_31_stored_entries():
    """46400 x 46400, fully dense: 2.15e9 stored entries, past the sign bit of a 32-bit index and half
    way to the format's limit of 2^32.  The encoding of a dense matrix is known in closed form (every
    code 0, row r starts at r * C, values = the matrix), so the GPU encoder is checked without the
    oracle's encoder; the product is checked against the oracle's dense product of the 464 distinct rows."""
    R = C = 46400
    blk = wl.bernoulli(464, C, 1.0, 0.02, 99, 1)            # 464 distinct rows, repeated 100 times
    assert ((blk & 0x7FFF) != 0).all()
    x = wl.x_vector(C, 99, 1)
    Wd = torch.from_numpy(blk.view(np.float16)).cuda().repeat(100, 1)
    m = M.encode_device(Wd)
    rep = m.get_report()
    assert rep.pad_nnz == R * C > 2 ** 31 and rep.nnz == R * C and rep.alloc_nnz == R * C
    vals, dels, rp = m.fetch_device()
    assert np.array_equal(rp.astype(np.int64), np.arange(R + 1, dtype=np.int64) * C)
    assert not dels.any()
    for row in (0, 463, 464, 23199, R - 1):
        assert np.array_equal(vals[row * C:(row + 1) * C], blk[row % 464]), row
    del vals, dels
    assert m.check_device() is None
    xd = to_dev(x)
    y = m.spmv(xd)
    torch.cuda.synchronize()
    y64, s64 = oracle.dense_matvec(blk, x)
    err = np.abs(y.float().cpu().numpy().astype(np.float64).reshape(100, 464) - y64[None, :])
    assert (err <= 1e-2 * s64[None, :] + 1e-3).all(), float(err.max())
    cols = m.columns_device()
    torch.cuda.synchronize()
    for row in (0, 1, 30000, R - 1):                          # entries beyond index 2^31 included
        assert torch.equal(cols[row * C:(row + 1) * C].cpu(), torch.arange(C, dtype=torch.int32)), row
    yd = M.dense_gemv(Wd, xd)
    torch.cuda.synchronize()
    err = np.abs(yd.float().cpu().numpy().astype(np.float64).reshape(100, 464) - y64[None, :])
    assert (err <= 1e-2 * s64[None, :] + 1e-3).all(), float(err.max())


# ------------------------------------------------------------------ many independent products in one call

def test_spmv_many_independent_products_eager_ordered_and_under_graph_capture():
    """macko_spmv_many deals grouped launches to the library's side streams.  Every product must equal
    the single-product call; work enqueued on the caller's stream before the call must be seen (the x
    vectors are written by a kernel on that stream right before) and work enqueued after it must see
    the results; captured into a graph, every replay must give the eager results again."""
    shapes = [(600, 2048, 0.5), (333, 1024, 0.6), (1200, 4096, 0.4), (64, 512, 0.5), (2000, 1536, 0.7)]
    mats, Ws = [], []
    for i in range(21):                                         # 21 products: three launches over three streams
        r, c, d = shapes[i % len(shapes)]
        W = wl.bernoulli(r, c, d, 0.02, 91, i)
        Ws.append(W)
        mats.append(M.encode(W, [4, 2, 4, 8, 4][i % 5]).to_device() if i % 7 else M.encode_fp8(wl.fp8_values_of(W)).to_device())
    xs_host = [wl.x_vector(W.shape[1], 91, i) for i, W in enumerate(Ws)]
    src = [to_dev(x) for x in xs_host]
    xs = [torch.zeros_like(s) for s in src]
    ys = [torch.empty(W.shape[0], dtype=torch.float16, device="cuda") for W in Ws]
    want = []
    for m, s in zip(mats, src):
        want.append(m.spmv(s).clone())
    torch.cuda.synchronize()
    many = M.SpmvMany(mats, xs, ys)
    main = torch.cuda.Stream()
    sums = [torch.zeros(1, dtype=torch.float32, device="cuda") for _ in ys]

    def enqueue():
        for x, s in zip(xs, src):                               # producers on the caller's stream ...
            x.copy_(s)
        many.launch(stream=torch.cuda.current_stream())
        for y, acc in zip(ys, sums):                            # ... and consumers after the call
            acc.copy_(y.float().abs().sum().reshape(1))

    with torch.cuda.stream(main):
        for rep in range(3):
            for x in xs:
                x.zero_()
            for y in ys:
                y.fill_(7.0)
            enqueue()
            main.synchronize()
            for i, (y, w, acc) in enumerate(zip(ys, want, sums)):
                assert torch.equal(y, w), f"eager rep {rep} product {i}"
                assert float(acc) == float(w.float().abs().sum()), f"consumer saw stale y, product {i}"
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=main):
            many.launch(stream=torch.cuda.current_stream())
        for rep in range(3):
            for y in ys:
                y.fill_(7.0)
            main.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for i, (y, w) in enumerate(zip(ys, want)):
                assert torch.equal(y, w), f"replay {rep} product {i}"
    # argument checks happen before anything is enqueued
    lib = M.load_library()
    assert lib.macko_spmv_many(-1, None, None, None, 0) < 0
    assert lib.macko_spmv_many(0, None, None, None, 0) == 0
    unbound = M.encode(Ws[0])
    bad = M.SpmvMany(mats[:9] + [unbound], xs[:9] + [xs[0]], ys[:9] + [ys[0]])
    assert bad.launch_raw(0) < 0


# ------------------------------------------------------------------ a chain of dependent products in one launch

def _chain_handles(shapes, seed, b_delta=4):
    return [M.encode(wl.half_row_matrix(r, c, 3000 + 10 * seed + i), b_delta).to_device()
            for i, (r, c) in enumerate(shapes)]


CHAINS = {
    # x of every product is the y of the one before: any stale or early read shows
    "tiny_4_phases": [(512, 512), (512, 512), (1024, 512), (512, 1024)],
    "ragged_3_phases": [(300, 777), (777, 300), (301, 777)],
    "layer_shapes": [(4096, 4096), (4096, 4096), (11008, 4096), (4096, 11008)],
    "eight_phases": [(640, 640)] * 8,
}


@pytest.mark.parametrize("b_delta", [4, 2])
@pytest.mark.parametrize("name", list(CHAINS))
def test_chain_of_dependent_products_equals_separate_launches(name, b_delta):
    """macko_spmv_chain: phase p + 1 reads what phase p wrote.  Per row the arithmetic is that of the
    wave-per-row kernel, so the results must equal those of separate launches in stream order bit
    for bit, and the first and last product are also checked against the oracle."""
    shapes = CHAINS[name]
    seed = sorted(CHAINS).index(name) + (10 if b_delta == 2 else 0)
    hs = _chain_handles(shapes, seed, b_delta)
    x0h = wl.x_vector(shapes[0][1], 7, seed)
    x0 = to_dev(x0h)
    M.set_tuning("spmv_kernel", 2)
    try:
        ref, x = [], x0
        for h in hs:
            x = h.spmv(x)
            ref.append(x)
        torch.cuda.synchronize()
    finally:
        M.set_tuning("spmv_kernel", 0)
    check_y(ref[0], wl.half_row_matrix(*shapes[0], 3000 + 10 * seed), x0h, name)
    ws = M.chain_workspace()
    ys = [torch.empty(h.rows, dtype=torch.float16, device="cuda") for h in hs]
    chain = M.SpmvChain([[(hs[i], x0 if i == 0 else ys[i - 1], ys[i])] for i in range(len(hs))], ws)
    for rep in range(10):
        for y in ys:
            y.fill_(float("nan"))
        chain.launch()
        torch.cuda.synchronize()
        assert chain.status() == (0, -1)
        for i, (y, r) in enumerate(zip(ys, ref)):
            assert torch.equal(y, r), f"{name} repetition {rep} phase {i}: {(y != r).sum().item()} rows differ"
    assert int(ws.to(torch.int32).abs().sum().item()) == 0          # the workspace is left zeroed
    last = len(hs) - 1
    check_y(ys[last], wl.half_row_matrix(*shapes[last], 3000 + 10 * seed + last),
            ref[last - 1].cpu().numpy().view(np.uint16), name + " last phase")


def test_chain_layer_step_as_the_bench_issues_it():
    """{q,k,v} -> {o} -> {gate,up} -> {down} of a Llama2-7B-shaped layer, several products per phase,
    against the four grouped launches of the same products, and against the oracle."""
    cases = list(wl.config2())
    h = {c.name.split("_")[1]: M.encode(c.W).to_device() for c in cases}
    x = {c.name.split("_")[1]: to_dev(c.x) for c in cases}
    hq, hg, hd = h["qkvo"], h["gate"], h["down"]
    xq, xg, xd = x["qkvo"], x["gate"], x["down"]

    def outs(m, n):
        return [torch.full((m.rows,), float("nan"), dtype=torch.float16, device="cuda") for _ in range(n)]
    yq, yo, yg, yd = outs(hq, 3), outs(hq, 1), outs(hg, 2), outs(hd, 1)
    phases = [[(hq, xq, y) for y in yq], [(hq, xq, yo[0])], [(hg, xg, y) for y in yg], [(hd, xd, yd[0])]]
    ws = M.chain_workspace()
    M.SpmvChain(phases, ws).launch()
    torch.cuda.synchronize()
    assert M.chain_status(ws) == (0, -1)
    for ph in phases:
        got = [y for _, _, y in ph]
        want = M.spmv_group([m for m, _, _ in ph], [xx for _, xx, _ in ph])
        torch.cuda.synchronize()
        for g, w in zip(got, want):
            assert torch.equal(g, w)
    for c, y in zip(cases, (yq[0], yg[1], yd[0])):
        check_y(y, c.W, c.x, "chain " + c.name)
    check_y(yo[0], cases[0].W, cases[0].x, "chain o")


def test_chain_gives_up_when_told_not_to_wait_and_recovers():
    """The bounded wait, forced from the host: with "chain_no_wait" a workgroup that finds the phase
    before unfinished gives up at once.  The launch still ends normally, the status call reports the
    phase, and the next chain on the same workspace runs as if nothing had happened."""
    hs = _chain_handles([(4096, 4096), (4096, 4096), (4096, 4096)], 5)
    x0 = to_dev(wl.x_vector(4096, 7, 5))
    ys = [torch.empty(4096, dtype=torch.float16, device="cuda") for _ in hs]
    ws = M.chain_workspace()
    chain = M.SpmvChain([[(hs[i], x0 if i == 0 else ys[i - 1], ys[i])] for i in range(3)], ws)
    chain.launch()
    torch.cuda.synchronize()
    assert chain.status() == (0, -1)
    good = [y.clone() for y in ys]
    M.set_tuning("chain_no_wait", 1)
    try:
        chain.launch()
        torch.cuda.synchronize()                      # returns: every workgroup has left
        st, phase = chain.status()
    finally:
        M.set_tuning("chain_no_wait", 0)
    assert st == M.MACKO_E_WAIT_EXPIRED and phase in (1, 2)
    assert torch.equal(ys[0], good[0])                # phase 0 waits for nothing and is complete
    assert chain.status() == (0, -1)                  # the record was cleared by the call that read it
    for y in ys:
        y.fill_(float("nan"))
    chain.launch()
    torch.cuda.synchronize()
    assert chain.status() == (0, -1)
    for y, g in zip(ys, good):
        assert torch.equal(y, g)
    assert int(ws.to(torch.int32).abs().sum().item()) == 0


def test_chain_argument_checks():
    lib = M.load_library()
    hs = _chain_handles([(512, 512)], 6)
    x = to_dev(wl.x_vector(512, 7, 6))
    y = torch.empty(512, dtype=torch.float16, device="cuda")
    ws = M.chain_workspace()
    # one phase of one product is an ordinary product
    M.SpmvChain([[(hs[0], x, y)]], ws).launch()
    torch.cuda.synchronize()
    assert torch.equal(y, spmv_case(wl.half_row_matrix(512, 512, 3060), wl.x_vector(512, 7, 6), spmv_kernel=2))
    # nine phases, seventeen products
    assert M.SpmvChain([[(hs[0], x, y)]] * 9, ws).launch_raw(0) == -3
    assert M.SpmvChain([[(hs[0], x, y)] * 3] * 6, ws).launch_raw(0) == -3
    assert M.SpmvChain([[(hs[0], x, y)] * 9], ws).launch_raw(0) == -1            # more than MACKO_MAX_GROUP in a phase
    # workspace: too small, misaligned, missing
    small = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    assert M.SpmvChain([[(hs[0], x, y)]], small).launch_raw(0) == -1
    big = torch.zeros(M.CHAIN_WORKSPACE_BYTES + 256, dtype=torch.uint8, device="cuda")
    assert M.SpmvChain([[(hs[0], x, y)]], big[8:]).launch_raw(0) == -1
    # 8-bit values and unbound handles are refused
    h8 = M.encode_fp8(wl.fp8_case(512, 512).W).to_device()
    assert M.SpmvChain([[(h8, x, y)]], ws).launch_raw(0) == -3
    assert M.SpmvChain([[(M.encode(wl.half_row_matrix(64, 64, 1)), x, y)]], ws).launch_raw(0) == -5
    empty = M.encode(np.zeros((64, 512), dtype=np.uint16)).to_device()
    assert M.SpmvChain([[(empty, x, torch.empty(64, dtype=torch.float16, device="cuda"))]], ws).launch_raw(0) == -3
    torch.cuda.synchronize()


# ------------------------------------------------------------------ a row depends on its own entries only

def _rows_ending_in_nonfinite(rows, cols, density, seed, fp8=False):
    """Every even row's last non-zero is an infinity or a NaN (a NaN only, for 8-bit values); odd rows are
    ordinary.  Most even rows end inside an 8-entry chunk that also holds the start of the next row."""
    W = wl.bernoulli(rows, cols, density, 0.02, 77, seed)
    if fp8:
        W = wl.fp8_values_of(W)
    for r in range(0, rows, 2):
        nz = np.flatnonzero(W[r])
        if nz.size:
            W[r, nz[-1]] = (0x7F if fp8 else (0x7C00, 0xFC00, 0x7E00)[(r // 2) % 3])
    return W


def _check_rows_independent(y_dev, W, x, what, dense=oracle.dense_matvec):
    y64, s64 = dense(W, x)
    y = y_dev.float().cpu().numpy().astype(np.float64)
    odd = np.arange(1, W.shape[0], 2)
    assert np.isfinite(y64[odd]).all()
    assert np.isfinite(y[odd]).all(), f"{what}: rows {odd[~np.isfinite(y[odd])][:8]} picked up a neighbour's inf/NaN"
    assert (np.abs(y[odd] - y64[odd]) <= REL_TOL * s64[odd] + ABS_TOL).all(), what
    even = np.arange(0, W.shape[0], 2)
    assert not np.isfinite(y[even]).any(), what
    assert np.array_equal(np.isnan(y[even]), np.isnan(y64[even])), what
    inf = even[np.isinf(y64[even])]
    assert np.array_equal(np.sign(y[inf]), np.sign(y64[inf])), what


@pytest.mark.parametrize("b_delta", [1, 2, 4, 8])
def test_inf_or_nan_at_the_end_of_a_row_stays_in_that_row(b_delta):
    """Section 4.4 makes y_i a function of row i alone.  The wave-per-row kernels load whole 8-entry chunks,
    so the lane that holds a row's start also holds the previous row's last entries; those must not reach
    this row's sum, not even as 0 * inf."""
    rows, cols = 130, 2048
    density = {1: 0.9, 2: 0.6, 4: 0.5, 8: 0.2}[b_delta]
    W = _rows_ending_in_nonfinite(rows, cols, density, b_delta)
    x = wl.x_vector(cols, 77, b_delta)
    x[x == 0] = 0x3C00
    for knobs in ({"spmv_kernel": 2}, {"spmv_kernel": 2, "spmv_step_align": 256},
                  {"spmv_kernel": 2, "spmv_step_align": 64, "spmv_block": 128, "spmv_rows_per_wg": 7},
                  {"spmv_kernel": 1, "spmv_lanes": 16}):
        y = spmv_case(W, x, b_delta=b_delta, **knobs)
        _check_rows_independent(y, W, x, f"b_delta {b_delta} {knobs}")
    # the small-batch kernel shares the pattern
    m = M.encode(W, b_delta).to_device()
    X = torch.stack([to_dev(x), to_dev(x)])
    Y = m.spmm(X)
    torch.cuda.synchronize()
    for b in range(2):
        _check_rows_independent(Y[b], W, x, f"spmm b_delta {b_delta} vector {b}")
    # and the chain (2- and 4-bit codes)
    if b_delta in (2, 4):
        y = torch.empty(rows, dtype=torch.float16, device="cuda")
        M.SpmvChain([[(m, to_dev(x), y)]]).launch()
        torch.cuda.synchronize()
        _check_rows_independent(y, W, x, f"chain b_delta {b_delta}")


def test_nan_at_the_end_of_a_row_stays_in_that_row_with_8_bit_values():
    rows, cols = 130, 2048
    W8 = _rows_ending_in_nonfinite(rows, cols, 0.5, 9, fp8=True)
    x = wl.x_vector(cols, 77, 9)
    x[x == 0] = 0x3C00
    for knobs in ({}, {"spmv_step_align": 256}):
        for k, v in knobs.items():
            M.set_tuning(k, v)
        try:
            y = M.encode_fp8(W8).to_device().spmv(to_dev(x))
            torch.cuda.synchronize()
        finally:
            for k in knobs:
                M.set_tuning(k, 0)
        _check_rows_independent(y, W8, x, f"8-bit values {knobs}", dense=oracle.dense_matvec8)


def test_chain_under_graph_capture_replays_like_eager():
    """macko_spmv_chain_static allocates nothing and records no memset, so it can be captured; every replay,
    with eager work and synchronisations between the replays, must reproduce the eager results, also when the
    chain's inputs changed in between (the graph holds pointers, not values)."""
    shapes = [(2048, 1536), (1536, 2048), (1024, 1536), (512, 1024)]
    hs = _chain_handles(shapes, 8)
    xa, xb = to_dev(wl.x_vector(1536, 7, 80)), to_dev(wl.x_vector(1536, 7, 81))
    x0 = torch.empty_like(xa)
    ys = [torch.empty(h.rows, dtype=torch.float16, device="cuda") for h in hs]
    chain = M.SpmvChain([[(hs[i], x0 if i == 0 else ys[i - 1], ys[i])] for i in range(4)])     # static scratch

    def eager(x):
        x0.copy_(x)
        chain.launch(stream=torch.cuda.current_stream())
        torch.cuda.synchronize()
        assert M.chain_status(None) == (0, -1)
        return [y.clone() for y in ys]

    main = torch.cuda.Stream()
    with torch.cuda.stream(main):
        want_a, want_b = eager(xa), eager(xb)        # also the first calls on this device: look-ups happen here
        assert not torch.equal(want_a[3], want_b[3])
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=main):
            chain.launch(stream=torch.cuda.current_stream())
        for rep, (x, want) in enumerate([(xa, want_a), (xb, want_b), (xb, want_b), (xa, want_a)]):
            x0.copy_(x)
            for y in ys:
                y.fill_(float("nan"))
            main.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for i, (y, w) in enumerate(zip(ys, want)):
                assert torch.equal(y, w), f"replay {rep} phase {i}"
            # eager work between replays: an ordinary product and another eager chain
            assert torch.equal(eager(x)[3], want[3])
        assert M.chain_status(None) == (0, -1)
