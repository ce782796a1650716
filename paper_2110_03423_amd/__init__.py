"""MI355X (gfx950) randomized SVD: thin Python binding over librsvd_gfx950.so.

Every step of the computation runs in the HIP kernels behind the C ABI declared
in include/rsvd.h; this package only marshals arguments.  PyTorch provides the
device memory and the stream.
"""
from .binding import (Rsvd, RsvdError, library_path, load_library, F32, F64,  # noqa: F401
                      JOB_S, JOB_SV, JOB_SUV, DEVICE_NONE)
