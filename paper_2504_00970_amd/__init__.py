"""MI355X-native SentenceKV hot path: HIP kernels behind a C ABI (include/sentencekv.h) plus a ctypes binding."""
from .binding import (Context, Desc, SkvError, EXPORTS, SKV_BF16, SKV_F32, SKV_FP8_E4M3, SKV_OK, SKV_EINVAL, SKV_ECAPACITY,
                      SKV_EHIP, SKV_ENOMEM, NOALLOC_SCRATCH_BYTES, decode_step_noalloc, dtype_code, lib_path)

__all__ = ["Context", "Desc", "SkvError", "EXPORTS", "SKV_BF16", "SKV_F32", "SKV_FP8_E4M3", "SKV_OK", "SKV_EINVAL", "SKV_ECAPACITY",
           "SKV_EHIP", "SKV_ENOMEM", "NOALLOC_SCRATCH_BYTES", "decode_step_noalloc", "dtype_code", "lib_path"]
