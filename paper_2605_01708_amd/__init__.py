"""SplitZip codec for MI355X: thin Python binding over libsplitzip.so.

Argument marshalling only.  PyTorch provides device memory and streams;
every step of the codec runs in the HIP kernels behind the C ABI declared
in include/splitzip.h.  There is no CPU fallback: if the library is missing
the import of this package fails.
"""
from .binding import (  # noqa: F401
    BF16,
    FP8_E5M2,
    STATUS_BAD_STREAM,
    STATUS_INTERNAL,
    STATUS_OVERFLOW,
    Codebook,
    CompressBatch,
    DecompressBatch,
    DeviceCodebook,
    SplitZipError,
    Workspace,
    calibrate,
    codebook_device,
    codebook_from_dec,
    codebook_from_hist,
    compress,
    compress_batch,
    compress_bound,
    compress_dcb,
    decompress,
    decompress_batch,
    decompress_dcb,
    fixed_bytes,
    histogram,
    lib,
    lib_path,
    new_sizes,
    new_sizes_array,
    read_sizes,
    read_sizes_array,
    total_bytes,
    traffic_probe,
    workspace_bytes,
)
