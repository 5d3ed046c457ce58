"""MACKO sparse matrix-vector product for AMD Instinct MI355X (gfx950).

Thin ctypes binding over ``libmacko.so`` (see ``include/macko.h``).  Every
arithmetic step runs inside the library's HIP kernels; this package only
marshals arguments.  PyTorch supplies device memory and streams.
"""
from .binding import (  # noqa: F401
    CHAIN_WORKSPACE_BYTES,
    MACKO_E_WAIT_EXPIRED,
    GemvGroup,
    MackoError,
    MackoMatrix,
    Report,
    SpmvChain,
    SpmvGroup,
    SpmvMany,
    chain_status,
    chain_workspace,
    dense_gemv,
    dense_gemv_group,
    encode,
    encode_device,
    encode_fp8,
    encode_device_fp8,
    get_tuning,
    library_path,
    load_library,
    set_tuning,
    spmv_group,
    status_string,
    storage_by_code_width,
    wrap_device,
    wrap_device_fp8,
)
