"""MI355X-native LazyTensor hot path: thin Python binding over the C ABI of liblt.so.

Everything that computes lives in the shared library (host C++ recorder / cache / lowering and
HIP kernels for gfx950).  This package only marshals arguments: it turns method calls on
`Tensor` objects into `lt_op` calls and exposes the barrier, fetch and the diagnostic dumps.
"""
from .lt import (Context, Tensor, LtError, BarrierInfo, load_library, library_path,  # noqa: F401
                 OPCODES, DTYPES)
