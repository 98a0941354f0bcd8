"""AdaFuse fused adapter switch for MI355X: thin ctypes binding over libadafuse.so.

Every step of the path runs in the HIP kernels behind the C ABI declared in
include/adafuse.h; this package only marshals arguments (torch tensors are
used for device memory and streams).  There is no CPU fallback: importing the
binding's entry points without the built library raises.
"""
from .binding import (  # noqa: F401
    GATE_SOFTMAX_OVER_TOPK,
    GATE_TOPK_OF_SOFTMAX,
    KERNEL_AUTO,
    KERNEL_GEMM,
    KERNEL_MFMA,
    KERNEL_VALU,
    MERGE,
    OPT_GEMM_FORM,
    OPT_GEMM_WAVES,
    OPT_KERNEL,
    OPT_MFMA_SHAPE,
    OPT_PANEL_KB,
    OPT_XCD_RUN,
    PROBE_READ_BASE,
    PROBE_ZERO_WORK,
    SWAP,
    UNMERGE,
    AdafuseError,
    Context,
    MatrixDesc,
    library_path,
    load_library,
    pregate,
)
