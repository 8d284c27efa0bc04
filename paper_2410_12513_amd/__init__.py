"""MI355X-native router-gated prefill/decode (FiRST).  Thin ctypes binding over libfirst.so;
every step of the path runs in the library's HIP kernels."""
from .binding import (FirstContext, FirstError, lib_path, load_library, op_gemv, op_gemm_nt, op_gemm_nt_f32a,
                      lora_merge, sample_top_k_static, EXPORTS, DTYPE_CODES)

__all__ = ["FirstContext", "FirstError", "lib_path", "load_library", "op_gemv", "op_gemm_nt", "op_gemm_nt_f32a",
           "lora_merge", "sample_top_k_static", "EXPORTS", "DTYPE_CODES"]
