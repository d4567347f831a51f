"""MI355X-native mixed-precision conv2d / matmul (int8 -> int32, fp16 -> fp32).

`unit` is the ctypes binding of libunit.so (HIP kernels behind a C ABI);
`workloads` holds shapes and seeded input generators only.
"""
from . import workloads  # noqa: F401
from . import unit  # noqa: F401
