"""MI355X-native batched JPEG -> model-input tensor preprocessing.

Thin ctypes binding of ``libprep.so`` (the C ABI declared in ``include/prep.h``).
All work happens in the library's HIP kernels; this module only marshals
arguments.  PyTorch is used by callers for device memory and streams.
"""
from .binding import (  # noqa: F401
    F16, F32, U8_NHWC, FILTER_ANTIALIAS, FILTER_BILINEAR, FLAG_FULL_RGB, FLAG_LARGE_WINDOWS, FLAG_SMOOTH_CHROMA, FLAG_TABLES_PER_WORKGROUP, OK, E_CORRUPT, E_HIP, E_INVALID_ARG, E_NOMEM, E_TOO_LARGE, E_UNSUPPORTED,
    AudioPreprocessor, BatchPolicy, ImageInfo, IntervalDesc, Preprocessor, PrepError, Server, build, lib, lib_path,
    parse_headers, interval_descriptors, resize_normalize_static, strerror,
)
