"""Token-wise RNN-T beam search on one MI355X: Python binding of libtbs.

The binding only marshals arguments (torch tensors -> device pointers, numpy
arrays -> host pointers); every step of the method runs in the HIP kernels of
the shared library.  There is no CPU fallback: importing this package without a
built libtbs.so raises.
"""

from .tbs import (  # noqa: F401
    Tbs,
    TbsError,
    load_library,
    gemm_bf16,
    LIB_PATH,
    BUF,
    KERNEL,
    EXPORTED_SYMBOLS,
)
