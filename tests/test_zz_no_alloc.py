"""macko_spmv_chain_static: the chain entry point that allocates nothing (its scratch is a static
device array of the library), against macko_spmv_chain with a caller-provided workspace, through
the C ABI, on two calls in a row, the second with a smaller input."""
import ctypes

import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
M = pytest.importorskip("paper_2511_13061_amd")


def _dev(a_u16):
    return torch.from_numpy(np.ascontiguousarray(a_u16).view(np.float16)).cuda()


def _chain_case(shapes, seed):
    Ws = [wl.half_row_matrix(r, c, 8100 + 10 * seed + i) for i, (r, c) in enumerate(shapes)]
    hs = [M.encode(W).to_device() for W in Ws]
    x0 = wl.x_vector(shapes[0][1], 11, seed)
    return Ws, hs, x0


def _run(lib, entry, hs, x0d, workspace):
    """One chain y0 = W0 x0, y1 = W1 y0, ... through the C ABI; returns the y tensors."""
    n = len(hs)
    ys = [torch.full((h.rows,), float("nan"), dtype=torch.float16, device="cuda") for h in hs]
    sizes = (ctypes.c_int * n)(*([1] * n))
    VP = ctypes.c_void_p * n
    handles = VP(*[h._h.value for h in hs])
    xs = VP(*([x0d.data_ptr()] + [y.data_ptr() for y in ys[:-1]]))
    yp = VP(*[y.data_ptr() for y in ys])
    stream = ctypes.c_void_p(int(torch.cuda.current_stream().cuda_stream))
    if entry == "static":
        st = lib.macko_spmv_chain_static(n, sizes, handles, xs, yp, stream)
    else:
        st = lib.macko_spmv_chain(n, sizes, handles, xs, yp, ctypes.c_void_p(workspace.data_ptr()),
                                  workspace.numel(), stream)
    assert st == 0, M.status_string(st)
    torch.cuda.synchronize()
    return ys


def test_chain_without_allocation_equals_chain_with_workspace_twice_in_a_row():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    lib = M.load_library()
    big = _chain_case([(4096, 4096), (11008, 4096), (4096, 11008)], 1)
    small = _chain_case([(512, 777), (300, 512)], 2)          # second call: smaller, ragged, most workgroups idle
    ws = torch.zeros(M.CHAIN_WORKSPACE_BYTES, dtype=torch.uint8, device="cuda")
    for Ws, hs, x0 in (big, small):
        x0d = _dev(x0)
        want = _run(lib, "workspace", hs, x0d, ws)
        got = _run(lib, "static", hs, x0d, None)
        for i, (g, w) in enumerate(zip(got, want)):
            assert torch.equal(g, w), f"phase {i}: {(g != w).sum().item()} rows differ"      # bit for bit
        # and both are right: first product against the oracle's dense product, the tolerance of the path
        y64, s64 = oracle.dense_matvec(Ws[0], x0)
        err = np.abs(got[0].float().cpu().numpy().astype(np.float64) - y64)
        assert (err <= 1e-2 * s64 + 1e-3).all()
        phase = ctypes.c_int(-2)
        assert lib.macko_chain_status(None, None, ctypes.byref(phase)) == 0 and phase.value == -1
    # sizes beyond the maximum are refused with a status, nothing is launched
    Ws, hs, x0 = small
    n = 9
    sizes = (ctypes.c_int * n)(*([1] * n))
    VP = ctypes.c_void_p * n
    y = torch.empty(512, dtype=torch.float16, device="cuda")
    st = lib.macko_spmv_chain_static(n, sizes, VP(*[hs[0]._h.value] * n), VP(*[_dev(x0).data_ptr()] * n),
                                     VP(*[y.data_ptr()] * n), None)
    assert st == -3 and M.status_string(st) == "unsupported"
