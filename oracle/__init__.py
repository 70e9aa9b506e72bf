"""CPU oracle for fp64 GEMM (test infrastructure; never imported by the product).

`gemm_f64_ref` and friends are thin ctypes wrappers over oracle/gemm_ref.c,
whose header states what is computed and which passage of the paper defines
it.  NumPy arrays are passed as host pointers plus leading dimensions.
"""
from .ref import (gemm_f64_ref, gemm_f64_ref_ijk, gemm_f64_absref, gemm_f32_ref, gemm_f32_ref_ijk,
                  gemm_f32_absref, ref_threads, set_ref_threads, ref_rows, abs_rows, gemm_general_ref,
                  general_scale, gemm_strided_ref, element_strides)

__all__ = ["gemm_f64_ref", "gemm_f64_ref_ijk", "gemm_f64_absref", "gemm_f32_ref", "gemm_f32_ref_ijk",
           "gemm_f32_absref", "ref_threads", "set_ref_threads", "ref_rows", "abs_rows", "gemm_general_ref", "general_scale",
           "gemm_strided_ref", "element_strides"]
