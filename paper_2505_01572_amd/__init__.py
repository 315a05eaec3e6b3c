"""pipeverify: the verification step of one PipeSpec pipeline stage on MI355X (gfx950).

Thin Python binding over the C ABI of libpipeverify.so (include/pipeverify.h).  Every step of
the path runs in the library's HIP kernels; Python only marshals arguments and uses torch
for device memory and streams.
"""
from .binding import (  # noqa: F401
    PVError, lib, Model, Cache, KINDS, PV_F32, PV_BF16, PATH_AUTO, PATH_VECTOR, PATH_MATRIX, PROF, calib_copy, calib_read, verify_batch,
)
