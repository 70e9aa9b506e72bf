"""Seeded synthetic matrices for the fp64 GEMM workloads.

This module holds input generation only; none of the GEMM arithmetic lives
here.  It serves the oracle-side tests and the HIP-side tests and benchmark
alike, so both see the same bits.

The paper's own workload (Section 1.3 and the driver in Section 2.1) is a
dense, unstructured 2088x2048x2048 (or 2048^3) row-major fp64 product whose
matrices are filled with the constant 1.0.  The stand-ins here keep that
shape class (dense, square-ish, row-major with an optional padded leading
dimension) and replace the constant by i.i.d. values so that indexing
mistakes cannot hide: uniform in [-1, 1) for the tolerance checks and uniform
integers in {-4..4} for the bit-exact checks.  `ones` reproduces the paper's
fill.

Values are a pure function of (seed, tag, i, j): a counter-based hash, so an
element does not depend on the leading dimension, on the order of generation
or on which rows are generated.
"""
from dataclasses import dataclass

import numpy as np

MASK64 = (1 << 64) - 1
TAG_A, TAG_B, TAG_C = 1, 2, 3

# Bit pattern written into leading-dimension padding: a quiet NaN that no
# arithmetic produces, so both "padding was read" (NaN leaks into C) and
# "padding was written" (pattern changed) are detectable.
PAD_BITS = 0x7FF8_5EED_0BAD_F00D
PAD_BITS32 = 0x7FC5_EED5  # the same idea for float32 buffers


def _mix_scalar(z: int) -> int:
    z = (z + 0x9E3779B97F4A7C15) & MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
    return z ^ (z >> 31)


def _mix_array(z: np.ndarray) -> np.ndarray:
    # SplitMix64 finaliser on uint64 arrays (arithmetic wraps modulo 2^64).
    z = z + np.uint64(0x9E3779B97F4A7C15)
    z ^= z >> np.uint64(30)
    z *= np.uint64(0xBF58476D1CE4E5B9)
    z ^= z >> np.uint64(27)
    z *= np.uint64(0x94D049BB133111EB)
    z ^= z >> np.uint64(31)
    return z


def _stream_key(seed: int, tag: int) -> int:
    return _mix_scalar((_mix_scalar(seed & MASK64) ^ (tag & MASK64)) & MASK64)


def hash_block(seed: int, tag: int, rows: np.ndarray, cols: np.ndarray) -> np.ndarray:
    """64-bit hash of every (row, col) pair; result shape (len(rows), len(cols))."""
    key = np.uint64(_stream_key(seed, tag))
    r = np.asarray(rows, dtype=np.uint64)[:, None]
    c = np.asarray(cols, dtype=np.uint64)[None, :]
    ctr = (r << np.uint64(32)) | c
    return _mix_array(ctr ^ key)


def values_uniform(h: np.ndarray) -> np.ndarray:
    """Top 53 bits -> multiples of 2^-52 in [-1, 1)."""
    return (h >> np.uint64(11)).astype(np.float64) * (2.0 ** -52) - 1.0


def values_int(h: np.ndarray) -> np.ndarray:
    """Integers uniform in {-4..4}, as float64."""
    return ((h >> np.uint64(11)) % np.uint64(9)).astype(np.float64) - 4.0


def values_uniform32(h: np.ndarray) -> np.ndarray:
    """Top 24 bits -> multiples of 2^-23 in [-1, 1), exactly representable in float32."""
    return ((h >> np.uint64(40)).astype(np.float64) * (2.0 ** -23) - 1.0).astype(np.float32)


_KINDS = ("uniform", "int", "ones", "zeros")


def fill(out: np.ndarray, seed: int, tag: int, kind: str, row0: int = 0,
         chunk_rows: int = 1024) -> np.ndarray:
    """Fill the 2-D float64 view `out` with element (row0 + i, j) of matrix `tag`."""
    assert kind in _KINDS
    rows, cols = out.shape
    if kind == "ones":
        out[...] = 1.0
        return out
    if kind == "zeros":
        out[...] = 0.0
        return out
    if out.dtype == np.float32:
        conv = values_uniform32 if kind == "uniform" else (lambda h: values_int(h).astype(np.float32))
    else:
        conv = values_uniform if kind == "uniform" else values_int
    cidx = np.arange(cols, dtype=np.uint64)
    for r in range(0, rows, chunk_rows):
        n = min(chunk_rows, rows - r)
        ridx = np.arange(row0 + r, row0 + r + n, dtype=np.uint64)
        out[r:r + n, :] = conv(hash_block(seed, tag, ridx, cidx))
    return out


def _signed(x: int) -> int:
    """The 64-bit pattern x as the signed integer torch's int64 holds for it."""
    x &= MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


def device_matrix(seed: int, tag: int, rows: int, cols: int, ld: int = None, kind: str = "uniform",
                  dtype=np.float64, device="cuda:0", chunk_rows: int = 2048):
    """The same matrix as `matrix`, bit for bit (sentinel padding included), generated on `device` with torch
    integer arithmetic: a (rows, ld) torch tensor.  int64 multiplication and addition wrap modulo 2^64 like the
    uint64 arithmetic of the NumPy path; logical right shifts are an arithmetic shift followed by a mask."""
    import torch
    assert kind in _KINDS
    ld = max(1, cols) if ld is None else ld
    assert ld >= max(1, cols)
    f32 = np.dtype(dtype) == np.float32
    tdt = torch.float32 if f32 else torch.float64
    idt = torch.int32 if f32 else torch.int64
    out = torch.empty((rows, ld), dtype=tdt, device=device)
    out.view(idt).fill_(PAD_BITS32 if f32 else _signed(PAD_BITS))   # PAD_BITS32 < 2^31 fits an int32 as it is
    view = out[:, :cols]
    if kind == "ones":
        view.fill_(1.0)
        return out
    if kind == "zeros":
        view.fill_(0.0)
        return out

    def lsr(z, n):
        return (z >> n) & ((1 << (64 - n)) - 1)

    key = _signed(_stream_key(seed, tag))
    c = torch.arange(cols, dtype=torch.int64, device=device)[None, :]
    for r0 in range(0, rows, chunk_rows):
        n = min(chunk_rows, rows - r0)
        r = torch.arange(r0, r0 + n, dtype=torch.int64, device=device)[:, None]
        z = ((r << 32) | c) ^ key
        z = z + _signed(0x9E3779B97F4A7C15)
        z = (z ^ lsr(z, 30)) * _signed(0xBF58476D1CE4E5B9)
        z = (z ^ lsr(z, 27)) * _signed(0x94D049BB133111EB)
        z = z ^ lsr(z, 31)
        if kind == "int":
            v = (lsr(z, 11) % 9).to(torch.float64) - 4.0
        elif f32:
            v = lsr(z, 40).to(torch.float64) * (2.0 ** -23) - 1.0
        else:
            v = lsr(z, 11).to(torch.float64) * (2.0 ** -52) - 1.0
        view[r0:r0 + n] = v.to(tdt)
    return out


def device_workload_inputs(w, seed: int = 0, integer: bool = False, dtype=np.float64, device="cuda:0"):
    """`workload_inputs` generated on the device: three (rows, ld) torch tensors holding the same bits."""
    kind = "int" if integer else "uniform"
    ckind = kind if w.c_kind == "uniform" else w.c_kind
    return (device_matrix(seed, TAG_A, w.M, w.K, w.lda, kind, dtype, device),
            device_matrix(seed, TAG_B, w.K, w.N, w.ldb, kind, dtype, device),
            device_matrix(seed, TAG_C, w.M, w.N, w.ldc, ckind, dtype, device))


def _bits_view(buf: np.ndarray):
    return (buf.view(np.uint32), np.uint32(PAD_BITS32)) if buf.dtype == np.float32 else (buf.view(np.uint64), np.uint64(PAD_BITS))


def padded(rows: int, cols: int, ld: int, pinned: bool = False, dtype=np.float64) -> np.ndarray:
    """A (rows, ld) buffer of `dtype` (float64 or float32) whose every element is the padding sentinel.

    With pinned=True the storage is page-locked host memory obtained from torch
    (a fresh allocation, never a registration of existing memory).
    """
    assert ld >= max(1, cols)
    dtype = np.dtype(dtype)
    if pinned:
        import torch
        tdt = torch.float32 if dtype == np.float32 else torch.float64
        t = torch.empty((max(rows, 1), ld), dtype=tdt, pin_memory=True)
        buf = t.numpy()[:rows]
    else:
        buf = np.empty((rows, ld), dtype=dtype)
    view, pad = _bits_view(buf)
    view[...] = pad
    return buf


def matrix(seed: int, tag: int, rows: int, cols: int, ld: int = None,
           kind: str = "uniform", dtype=np.float64):
    """Return (buffer, view): buffer is (rows, ld) with sentinel padding, view = buffer[:, :cols]."""
    ld = max(1, cols) if ld is None else ld
    buf = padded(rows, cols, ld, dtype=dtype)
    view = buf[:, :cols]
    fill(view, seed, tag, kind)
    return buf, view


def padding_intact(buf: np.ndarray, cols: int) -> bool:
    """True when every element at column >= cols still holds the sentinel bits."""
    if buf.shape[1] == cols:
        return True
    view, pad = _bits_view(buf)
    return bool(np.all(view[:, cols:] == pad))


@dataclass(frozen=True)
class Workload:
    name: str
    M: int
    N: int
    K: int
    lda: int
    ldb: int
    ldc: int
    c_kind: str  # how C is initialised for the uniform variant

    @property
    def flops(self) -> float:
        return 2.0 * self.M * self.N * self.K

    @property
    def algorithmic_bytes(self) -> float:
        # read A, B and C once, write C once
        return 8.0 * (self.M * self.K + self.K * self.N + 2 * self.M * self.N)


# The five benchmark/parity configurations.
WORKLOADS = {
    "c0_256": Workload("c0_256", 256, 256, 256, 256, 256, 256, "uniform"),
    "c1_2048": Workload("c1_2048", 2048, 2048, 2048, 2048, 2048, 2048, "uniform"),
    "c2_edge": Workload("c2_edge", 2088, 2049, 2047, 2056, 2064, 2064, "uniform"),
    "c3_8192": Workload("c3_8192", 8192, 8192, 8192, 8192, 8192, 8192, "zeros"),
    "c4_rankk": Workload("c4_rankk", 16384, 16384, 256, 256, 16384, 16384, "uniform"),
}


def workload_inputs(w: Workload, seed: int = 0, integer: bool = False, dtype=np.float64):
    """(Abuf, Bbuf, Cbuf) padded host buffers for a workload; logical parts are [:, :K] etc."""
    kind = "int" if integer else "uniform"
    ckind = kind if w.c_kind == "uniform" else w.c_kind
    Abuf, _ = matrix(seed, TAG_A, w.M, w.K, w.lda, kind, dtype)
    Bbuf, _ = matrix(seed, TAG_B, w.K, w.N, w.ldb, kind, dtype)
    Cbuf, _ = matrix(seed, TAG_C, w.M, w.N, w.ldc, ckind, dtype)
    return Abuf, Bbuf, Cbuf


def sample_rows(M: int, count: int, seed: int = 0, period: int = 128) -> np.ndarray:
    """Rows to verify at sizes where the oracle cannot do the whole matrix.

    Always includes the first and last row and the rows on both sides of every
    multiple-of-`period` boundary near the start, middle and end, then fills up
    with hashed pseudo-random rows.  Sorted, unique.
    """
    fixed = {0, M - 1}
    for base in (0, (M // 2 // period) * period, ((M - 1) // period) * period):
        for d in (-1, 0, 1, period // 2 - 1, period // 2, period - 1):
            r = base + d
            if 0 <= r < M:
                fixed.add(r)
    rows = set(fixed)
    ctr = 0
    while len(rows) < min(count, M):
        rows.add(_mix_scalar(_stream_key(seed, 99) ^ ctr) % M)
        ctr += 1
    return np.array(sorted(rows), dtype=np.int64)
