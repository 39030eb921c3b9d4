"""MI355X-native hot path of the distributed embedding lookup of bounded-lag-synchronous
DLRM inference: a HIP library (libbls.so, C ABI in include/bls.h) and this thin ctypes
binding.  Every step of the path runs in the library's kernels; there is no fallback."""
from .bls import (  # noqa: F401
    BLS_OK, BLS_EINVAL, BLS_ERANGE, BLS_ENOSPC, BLS_ERING_FULL, BLS_ERING_EMPTY, BLS_EORDER, BLS_EHIP,
    BLS_FP32, BLS_FP16, BLS_U8_ROWQ, BLS_F8_ROWQ, BLS_TABLE_WISE, BLS_ROW_WISE, BLS_ACT_NONE, BLS_ACT_RELU, BLS_ACT_SIGMOID,
    BlsError, Context, lib, lib_path, EXPORTS,
)
