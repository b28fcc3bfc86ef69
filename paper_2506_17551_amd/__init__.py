"""MI355X-native gradient compression before aggregation (paper Sec. III.B):
error-feedback accumulate, exact magnitude top-k, per-block int8 codes, and the
matching decompress-and-sum. The compute lives in libgradcomp.so (hand-written
HIP for gfx950, C ABI in include/gradcomp.h); this package only marshals
arguments. PyTorch supplies device memory and streams."""
from .binding import (CompressedBuf, Context, GradCompError, compress, compress_multi,  # noqa: F401
                      decompress_sum, decompress_sum_static, decompress_sum_multi, decompress_sum_weighted, decompress_apply,
                      compress_rows, decompress_sum_rows, compress_dense, decompress_sum_dense, decompress_apply_dense, k_from_density, num_scales, num_code_bytes, GC_CODEC_INT8, GC_CODEC_SIGN1,
                      sync_status, last_stats)
