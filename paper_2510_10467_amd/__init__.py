"""MI355X-native AnyBCQ inference kernels (bit-plane BCQ product), gfx950 only.

The product path is the HIP library ``libbcq_hip.so`` behind the C ABI of
``include/bcq.h``; this package is its thin Python binding.
"""
from .binding import (BcqError, bench_fp16_gemv, bench_issue_probe, bench_stream_read, bcq_gemm_mixed, bcq_gemv, bcq_gemv_multi, bcq_pack, bcq_quantize, bcq_unpack, last_kernel, lib,  # noqa: F401
                      select_dequant_shape, select_kernel)
