"""Thin ctypes binding of libgemm_f64.so (see include/gemm_f64.h).

Argument marshalling only: every function forwards to the C entry point of the
same name.  Device buffers may be given as torch tensors (their data_ptr is
used) or as integer addresses.  There is no fallback of any kind: if the
library has not been built, loading raises.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgemm_f64.so")

_lib = None


class GemmF64Error(RuntimeError):
    def __init__(self, code, text):
        super().__init__("gemm_f64 error %d: %s" % (code, text))
        self.code = code


def load():
    """Load libgemm_f64.so; raises if it is missing (build it with __graft_entry__.build())."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s not found: the HIP library is not built (run `python -c 'import __graft_entry__ as g; g.build()'`); "
            "there is no CPU fallback" % LIB_PATH)
    # PyTorch ships its own copy of the HIP runtime.  When it is present it must be loaded first, so that this
    # library binds to the same runtime as the tensors and streams it is handed; two runtimes in one process do not
    # share streams or loaded kernels, and launches fail.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(LIB_PATH)
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    lib.gemm_f64.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, vp]
    lib.gemm_f64.restype = ci
    lib.gemm_f64_ex.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, vp, ci]
    lib.gemm_f64_ex.restype = ci
    lib.gemm_f64_variant_count.argtypes = []
    lib.gemm_f64_variant_count.restype = ci
    lib.gemm_f64_variant_name.argtypes = [ci]
    lib.gemm_f64_variant_name.restype = ctypes.c_char_p
    lib.gemm_f64_choose_variant.argtypes = [i64, i64, i64, ci]
    lib.gemm_f64_choose_variant.restype = ci
    lib.gemm_f64_tile_of_block.argtypes = [i64, i64, i64, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    lib.gemm_f64_tile_of_block.restype = ci
    lib.gemm_f64_strerror.argtypes = [ci]
    lib.gemm_f64_strerror.restype = ctypes.c_char_p
    lib.gemm_f64_version.argtypes = []
    lib.gemm_f64_version.restype = ci
    lib.gemm_f64_set_epilogue_mode.argtypes = [ci]
    lib.gemm_f64_set_epilogue_mode.restype = ci
    lib.gemm_f64_build_id.argtypes = []
    lib.gemm_f64_build_id.restype = ctypes.c_char_p
    lib.gemm_f32.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, vp]
    lib.gemm_f32.restype = ci
    lib.gemm_f32_ex.argtypes = [i64, i64, i64, vp, i64, vp, i64, vp, i64, vp, ci]
    lib.gemm_f32_ex.restype = ci
    lib.gemm_f32_variant_count.argtypes = []
    lib.gemm_f32_variant_count.restype = ci
    lib.gemm_f32_variant_name.argtypes = [ci]
    lib.gemm_f32_variant_name.restype = ctypes.c_char_p
    lib.gemm_f32_choose_variant.argtypes = [i64, i64, i64, ci]
    lib.gemm_f32_choose_variant.restype = ci
    for fn in (lib.gemm_f64_choose_variant_general, lib.gemm_f32_choose_variant_general):
        fn.argtypes = [ci, ci, i64, i64, i64, ci]
        fn.restype = ci
    for fn in (lib.gemm_f64_mfma_probe, lib.gemm_f32_mfma_probe):
        fn.argtypes = [i64, vp, i64, vp, ctypes.POINTER(ctypes.c_double)]
        fn.restype = ci
    ip = ctypes.POINTER(ci)
    for fn in (lib.gemm_f64_split_k_plan, lib.gemm_f32_split_k_plan):
        fn.argtypes = [ci, ci, i64, i64, i64, ci, i64, ip, ip, ip]
        fn.restype = ci
    for fn in (lib.gemm_f64_tail_split_plan, lib.gemm_f32_tail_split_plan):
        fn.argtypes = [ci, ci, i64, i64, i64, ci, i64, ip, ip, ip, ip]
        fn.restype = ci
    for fn in (lib.gemm_f64_split_k_workspace_bytes, lib.gemm_f32_split_k_workspace_bytes):
        fn.argtypes = [ci, ci, i64, i64, i64, ci]
        fn.restype = i64
    cd, cf = ctypes.c_double, ctypes.c_float
    lib.gemm_f64_general_ws.argtypes = [ci, ci, i64, i64, i64, cd, vp, i64, vp, i64, cd, vp, i64, vp, i64, vp]
    lib.gemm_f64_general_ws.restype = ci
    lib.gemm_f32_general_ws.argtypes = [ci, ci, i64, i64, i64, cf, vp, i64, vp, i64, cf, vp, i64, vp, i64, vp]
    lib.gemm_f32_general_ws.restype = ci
    lib.gemm_f64_general.argtypes = [ci, ci, i64, i64, i64, cd, vp, i64, vp, i64, cd, vp, i64, vp]
    lib.gemm_f64_general.restype = ci
    lib.gemm_f64_general_ex.argtypes = [ci, ci, i64, i64, i64, cd, vp, i64, vp, i64, cd, vp, i64, vp, ci]
    lib.gemm_f64_general_ex.restype = ci
    lib.gemm_f32_general.argtypes = [ci, ci, i64, i64, i64, cf, vp, i64, vp, i64, cf, vp, i64, vp]
    lib.gemm_f32_general.restype = ci
    lib.gemm_f32_general_ex.argtypes = [ci, ci, i64, i64, i64, cf, vp, i64, vp, i64, cf, vp, i64, vp, ci]
    lib.gemm_f32_general_ex.restype = ci
    lib.gemm_f64_device_peak.argtypes = [ip, ip, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.gemm_f64_device_peak.restype = ci
    lp = ctypes.POINTER(i64)
    lib.gemm_f64_strided_path.argtypes = [i64] * 9 + [ip, ip, ip, lp, lp, lp, lp, lp, lp]
    lib.gemm_f64_strided_path.restype = ci
    lib.gemm_f64_general_static.argtypes = [ci, ci, i64, i64, i64, cd, vp, i64, vp, i64, cd, vp, i64, vp]
    lib.gemm_f64_general_static.restype = ci
    lib.gemm_f64_strided.argtypes = [i64, i64, i64, cd, vp, i64, i64, vp, i64, i64, cd, vp, i64, i64, vp]
    lib.gemm_f64_strided.restype = ci
    lib.gemm_f32_strided.argtypes = [i64, i64, i64, cf, vp, i64, i64, vp, i64, i64, cf, vp, i64, i64, vp]
    lib.gemm_f32_strided.restype = ci
    _lib = lib
    return lib


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def gemm_f64_strerror(code: int) -> str:
    return load().gemm_f64_strerror(int(code)).decode()


def _check(code):
    if code != 0:
        raise GemmF64Error(code, gemm_f64_strerror(code))


def gemm_f64(M, N, K, A, lda, B, ldb, C, ldc, stream=None):
    """Enqueue C += A @ B (device pointers, row-major, leading dimensions in elements)."""
    _check(load().gemm_f64(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, _stream(stream)))


def gemm_f64_ex(M, N, K, A, lda, B, ldb, C, ldc, stream=None, variant=-1):
    """Same, with an explicit kernel variant (-1 = automatic)."""
    _check(load().gemm_f64_ex(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, _stream(stream), int(variant)))


def gemm_f64_raw(M, N, K, A, lda, B, ldb, C, ldc, stream=0, variant=-1) -> int:
    """Return the raw status code instead of raising (for error-path tests)."""
    return int(load().gemm_f64_ex(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, stream, int(variant)))


def gemm_f64_variant_count() -> int:
    return int(load().gemm_f64_variant_count())


def gemm_f64_variant_name(variant: int):
    s = load().gemm_f64_variant_name(int(variant))
    return None if s is None else s.decode()


def gemm_f64_choose_variant(M, N, K, num_cu=256) -> int:
    return int(load().gemm_f64_choose_variant(M, N, K, int(num_cu)))


def gemm_f64_choose_variant_general(transa, transb, M, N, K, num_cu=256) -> int:
    return int(load().gemm_f64_choose_variant_general(int(transa), int(transb), M, N, K, int(num_cu)))


def gemm_f32_choose_variant_general(transa, transb, M, N, K, num_cu=256) -> int:
    return int(load().gemm_f32_choose_variant_general(int(transa), int(transb), M, N, K, int(num_cu)))


def gemm_f64_tile_of_block(block, tiles_m, tiles_n):
    tm, tn = ctypes.c_int64(-1), ctypes.c_int64(-1)
    _check(load().gemm_f64_tile_of_block(block, tiles_m, tiles_n, ctypes.byref(tm), ctypes.byref(tn)))
    return int(tm.value), int(tn.value)


def gemm_f64_version() -> int:
    return int(load().gemm_f64_version())


def gemm_f64_set_epilogue_mode(mode: int) -> int:
    """Diagnostic switch: 0 automatic, 1 load-add-store, 2 additions in memory; returns the previous mode."""
    rc = int(load().gemm_f64_set_epilogue_mode(int(mode)))
    _check(rc if rc < 0 else 0)
    return rc


def gemm_f64_build_id() -> str:
    return load().gemm_f64_build_id().decode()


# ---- single precision (include/gemm_f32.h) ------------------------------------------------------

def gemm_f32(M, N, K, A, lda, B, ldb, C, ldc, stream=None):
    """Enqueue float C += A @ B (device pointers, row-major, leading dimensions in elements)."""
    _check(load().gemm_f32(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, _stream(stream)))


def gemm_f32_ex(M, N, K, A, lda, B, ldb, C, ldc, stream=None, variant=-1):
    _check(load().gemm_f32_ex(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, _stream(stream), int(variant)))


def gemm_f32_raw(M, N, K, A, lda, B, ldb, C, ldc, stream=0, variant=-1) -> int:
    return int(load().gemm_f32_ex(M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, stream, int(variant)))


def gemm_f32_variant_count() -> int:
    return int(load().gemm_f32_variant_count())


def gemm_f32_variant_name(variant: int):
    s = load().gemm_f32_variant_name(int(variant))
    return None if s is None else s.decode()


def gemm_f32_choose_variant(M, N, K, num_cu=256) -> int:
    return int(load().gemm_f32_choose_variant(M, N, K, int(num_cu)))


# ---- C <- alpha * op(A) op(B) + beta * C ---------------------------------------------------------

def gemm_f64_general(transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream=None):
    """Enqueue C <- alpha * op(A) @ op(B) + beta * C (double; A is K x M when transa, B is N x K when transb)."""
    _check(load().gemm_f64_general(int(transa), int(transb), M, N, K, alpha, _ptr(A), lda, _ptr(B), ldb, beta,
                                   _ptr(C), ldc, _stream(stream)))


def gemm_f64_general_ex(transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream=None, variant=-1):
    _check(load().gemm_f64_general_ex(int(transa), int(transb), M, N, K, alpha, _ptr(A), lda, _ptr(B), ldb, beta,
                                      _ptr(C), ldc, _stream(stream), int(variant)))


def gemm_f64_general_raw(transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream=0, variant=-1) -> int:
    return int(load().gemm_f64_general_ex(int(transa), int(transb), M, N, K, alpha, _ptr(A), lda, _ptr(B), ldb, beta,
                                          _ptr(C), ldc, stream, int(variant)))


def gemm_f32_general(transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream=None):
    """The float counterpart of gemm_f64_general."""
    _check(load().gemm_f32_general(int(transa), int(transb), M, N, K, alpha, _ptr(A), lda, _ptr(B), ldb, beta,
                                   _ptr(C), ldc, _stream(stream)))


def gemm_f32_general_ex(transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream=None, variant=-1):
    _check(load().gemm_f32_general_ex(int(transa), int(transb), M, N, K, alpha, _ptr(A), lda, _ptr(B), ldb, beta,
                                      _ptr(C), ldc, _stream(stream), int(variant)))


def gemm_f32_general_raw(transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream=0, variant=-1) -> int:
    return int(load().gemm_f32_general_ex(int(transa), int(transb), M, N, K, alpha, _ptr(A), lda, _ptr(B), ldb, beta,
                                          _ptr(C), ldc, stream, int(variant)))


def gemm_f64_mfma_probe(iterations, sink, sink_elems, stream=None) -> float:
    """Enqueue the MFMA-only probe (double); returns the floating-point operations of the launch."""
    flops = ctypes.c_double(0.0)
    _check(load().gemm_f64_mfma_probe(int(iterations), _ptr(sink), int(sink_elems), _stream(stream), ctypes.byref(flops)))
    return float(flops.value)


def gemm_f32_mfma_probe(iterations, sink, sink_elems, stream=None) -> float:
    flops = ctypes.c_double(0.0)
    _check(load().gemm_f32_mfma_probe(int(iterations), _ptr(sink), int(sink_elems), _stream(stream), ctypes.byref(flops)))
    return float(flops.value)


# ---- split K with a caller-provided workspace --------------------------------------------------

def gemm_f64_general_ws(transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, workspace, workspace_bytes, stream=None):
    """gemm_f64_general with a device workspace on offer (the library may split the k range)."""
    _check(load().gemm_f64_general_ws(int(transa), int(transb), M, N, K, alpha, _ptr(A), lda, _ptr(B), ldb, beta,
                                      _ptr(C), ldc, _ptr(workspace), int(workspace_bytes), _stream(stream)))


def gemm_f64_general_static(transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, stream=None):
    """gemm_f64_general_ws on the library's own fixed scratch buffer: allocates nothing."""
    _check(load().gemm_f64_general_static(int(transa), int(transb), M, N, K, alpha, _ptr(A), lda, _ptr(B), ldb, beta,
                                          _ptr(C), ldc, _stream(stream)))


STATIC_SCRATCH_BYTES = 64 << 20   # GEMM_F64_STATIC_SCRATCH_BYTES


def gemm_f32_general_ws(transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc, workspace, workspace_bytes, stream=None):
    _check(load().gemm_f32_general_ws(int(transa), int(transb), M, N, K, alpha, _ptr(A), lda, _ptr(B), ldb, beta,
                                      _ptr(C), ldc, _ptr(workspace), int(workspace_bytes), _stream(stream)))


def gemm_f64_device_peak():
    """(compute units, clock in kHz, FP64 MFMA peak, FP32 MFMA peak in TFLOP/s) of the current device."""
    cus, khz, p64, p32 = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_double(0), ctypes.c_double(0)
    _check(load().gemm_f64_device_peak(ctypes.byref(cus), ctypes.byref(khz), ctypes.byref(p64), ctypes.byref(p32)))
    return cus.value, khz.value, p64.value, p32.value


def gemm_f64_strided_path(M, N, K, rsa, csa, rsb, csb, rsc, csc):
    """(kind, swapped, transa, transb, lda, ldb, ldc, es_a, es_b, es_c) of the problem that a strided call runs (kind 1:
    transposed signature, 2: sampled mode); raises for sizes or strides that gemm_f64_strided rejects."""
    sw, ta, tb = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_int(0)
    out = [ctypes.c_int64(0) for _ in range(6)]
    rc = load().gemm_f64_strided_path(M, N, K, rsa, csa, rsb, csb, rsc, csc, ctypes.byref(sw), ctypes.byref(ta), ctypes.byref(tb),
                                      *[ctypes.byref(x) for x in out])
    if rc < 0:
        _check(rc)
    return (rc, bool(sw.value), ta.value, tb.value) + tuple(x.value for x in out)


def gemm_f64_strided(M, N, K, alpha, A, rsa, csa, B, rsb, csb, beta, C, rsc, csc, stream=None):
    """Enqueue C <- alpha * A @ B + beta * C (double) with X(r, c) = X[r * rs + c * cs] for every operand."""
    _check(load().gemm_f64_strided(M, N, K, alpha, _ptr(A), rsa, csa, _ptr(B), rsb, csb, beta, _ptr(C), rsc, csc,
                                   _stream(stream)))


def gemm_f32_strided(M, N, K, alpha, A, rsa, csa, B, rsb, csb, beta, C, rsc, csc, stream=None):
    _check(load().gemm_f32_strided(M, N, K, alpha, _ptr(A), rsa, csa, _ptr(B), rsb, csb, beta, _ptr(C), rsc, csc,
                                   _stream(stream)))


def gemm_f64_strided_raw(M, N, K, alpha, A, rsa, csa, B, rsb, csb, beta, C, rsc, csc, stream=0) -> int:
    return int(load().gemm_f64_strided(M, N, K, alpha, _ptr(A), rsa, csa, _ptr(B), rsb, csb, beta, _ptr(C), rsc, csc, stream))


def gemm_f32_strided_raw(M, N, K, alpha, A, rsa, csa, B, rsb, csb, beta, C, rsc, csc, stream=0) -> int:
    return int(load().gemm_f32_strided(M, N, K, alpha, _ptr(A), rsa, csa, _ptr(B), rsb, csb, beta, _ptr(C), rsc, csc, stream))


def _plan(fn, transa, transb, M, N, K, num_cu, workspace_bytes):
    v, s, c = ctypes.c_int(-1), ctypes.c_int(-1), ctypes.c_int(-1)
    _check(fn(int(transa), int(transb), M, N, K, int(num_cu), int(workspace_bytes), ctypes.byref(v), ctypes.byref(s), ctypes.byref(c)))
    return int(v.value), int(s.value), int(c.value)


def gemm_f64_split_k_plan(transa, transb, M, N, K, num_cu=256, workspace_bytes=2 ** 62):
    """(variant, splits, k_chunk) that gemm_f64_general_ws uses for these arguments."""
    return _plan(load().gemm_f64_split_k_plan, transa, transb, M, N, K, num_cu, workspace_bytes)


def gemm_f32_split_k_plan(transa, transb, M, N, K, num_cu=256, workspace_bytes=2 ** 62):
    return _plan(load().gemm_f32_split_k_plan, transa, transb, M, N, K, num_cu, workspace_bytes)


def _tail_plan(fn, transa, transb, M, N, K, num_cu, workspace_bytes):
    v, t, s, c = (ctypes.c_int(-1) for _ in range(4))
    _check(fn(int(transa), int(transb), M, N, K, int(num_cu), int(workspace_bytes), ctypes.byref(v), ctypes.byref(t),
              ctypes.byref(s), ctypes.byref(c)))
    return int(v.value), int(t.value), int(s.value), int(c.value)


def gemm_f64_tail_split_plan(transa, transb, M, N, K, num_cu=256, workspace_bytes=2 ** 62):
    """(variant, tail tiles, slices per tail tile, slice length) of a call with this much workspace; 0 tiles: no tail split."""
    return _tail_plan(load().gemm_f64_tail_split_plan, transa, transb, M, N, K, num_cu, workspace_bytes)


def gemm_f32_tail_split_plan(transa, transb, M, N, K, num_cu=256, workspace_bytes=2 ** 62):
    return _tail_plan(load().gemm_f32_tail_split_plan, transa, transb, M, N, K, num_cu, workspace_bytes)


def gemm_f64_split_k_workspace_bytes(transa, transb, M, N, K, num_cu=256) -> int:
    return int(load().gemm_f64_split_k_workspace_bytes(int(transa), int(transb), M, N, K, int(num_cu)))


def gemm_f32_split_k_workspace_bytes(transa, transb, M, N, K, num_cu=256) -> int:
    return int(load().gemm_f32_split_k_workspace_bytes(int(transa), int(transb), M, N, K, int(num_cu)))


def variant_index(name: str) -> int:
    for v in range(gemm_f64_variant_count()):
        if gemm_f64_variant_name(v) == name:
            return v
    raise KeyError(name)
