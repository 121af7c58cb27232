"""MI355X-native BalanceKV hot path (arXiv 2502.07861): HIP kernels behind a C ABI + ctypes binding."""
from .binding import (BKV_BF16, BKV_CENTER_KEYS, BKV_F32, BKV_SET_DENOMINATOR, BKV_SET_NUMERATOR, BKV_STRICT_HALF,
                      BKV_STREAM_DEN_FULL, BKV_STREAM_NO_REGION, BKV_STREAM_NUM_FULL, BKV_VALUE_GRAM, BkvError, Cache, Stream,
                      attend_kv, attend_sets, balancekv_sets, bkv_params, compress_block,
                      kernel_weights, lib, make_params, merge_reduce, merge_reduce_protected, uniform_bits)

__all__ = ["BKV_BF16", "BKV_CENTER_KEYS", "BKV_F32", "BKV_SET_DENOMINATOR", "BKV_SET_NUMERATOR", "BKV_STRICT_HALF",
           "BKV_STREAM_DEN_FULL", "BKV_STREAM_NO_REGION", "BKV_STREAM_NUM_FULL", "BKV_VALUE_GRAM", "BkvError", "Cache", "Stream", "attend_kv", "attend_sets", "balancekv_sets", "bkv_params", "compress_block", "kernel_weights", "lib", "make_params", "merge_reduce",
           "merge_reduce_protected", "uniform_bits"]
