"""C <- alpha * A B + beta * C on operands addressed through two strides each, on the GPU against its CPU
oracle, through the C ABI, in both precisions (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2003_00532_amd import binding

import gpu_util
import pins
import pins_general as pg
import pins_strided as ps

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
GUARD = 32   # sentinel elements on either side of every device buffer
DTYPES = [np.float64, np.float32]


def _span(view):
    """The view's memory from its first to its last element as a flat writable array (strides are positive)."""
    sz = view.dtype.itemsize
    rs, cs = oracle.element_strides(view)
    n = (view.shape[0] - 1) * rs + (view.shape[1] - 1) * cs + 1
    return np.lib.stride_tricks.as_strided(view, shape=(n,), strides=(sz,))


def device_call(alpha, A, B, beta, C):
    """Copy the memory under the three views to guarded device buffers, run the strided entry point on the
    same strides, copy all of C's memory back.  A and B must come back unchanged and no guard may be written."""
    f32 = C.dtype == np.float32
    M, N = C.shape
    K = A.shape[1]
    held = []
    for v in (A, B, C):
        if v.size == 0:
            held.append((None, torch.full((2 * GUARD + 1,), float("nan"), dtype=torch.float32 if f32 else torch.float64, device=DEV), None))
            continue
        flat = _span(v)
        host = torch.full((flat.size + 2 * GUARD,), float("nan"), dtype=torch.float32 if f32 else torch.float64)
        host[GUARD:GUARD + flat.size] = torch.from_numpy(flat.copy())
        held.append((flat, host.to(DEV), host))
    sz = C.dtype.itemsize
    ptr = lambda h: h[1].data_ptr() + GUARD * sz
    (rsa, csa), (rsb, csb), (rsc, csc) = (oracle.element_strides(v) for v in (A, B, C))
    fn = binding.gemm_f32_strided if f32 else binding.gemm_f64_strided
    fn(M, N, K, float(alpha), ptr(held[0]), rsa, csa, ptr(held[1]), rsb, csb, float(beta), ptr(held[2]), rsc, csc)
    torch.cuda.synchronize()
    iv = torch.int32 if f32 else torch.int64
    for name, (flat, dev, host) in zip("ABC", held):
        got = dev.cpu()
        n = 0 if flat is None else flat.size
        assert bool(torch.isnan(got[:GUARD]).all()) and bool(torch.isnan(got[GUARD + n:]).all()), "memory around %s was written" % name
        if flat is None:
            continue
        if name == "C":
            flat[...] = got[GUARD:GUARD + n].numpy()
        else:
            assert torch.equal(got.view(iv), host.view(iv)), "%s was written" % name


# the pins that hold for any order of summation (the others fix the rounding of every partial sum, and the
# device adds in the matrix unit's order)
ORDER_FREE = [p for p in ps.ALL_PINS if p is not ps.pin_strided_rounded_sequence]
ORDER_FREE_GENERAL = [pg.pin_general_tiny_exact, pg.pin_general_all_ones, pg.pin_general_one_hot, pg.pin_general_unread_operands,
                      pg.pin_general_integer_exact, pg.pin_general_error_bound]


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("pin", ORDER_FREE, ids=lambda p: p.__name__)
def test_strided_pins_on_the_device(gpu_device, pin, dtype):
    with pins.precision(dtype):
        pin(device_call)


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("c_layout", ["row", "col", "row_step2"])
@pytest.mark.parametrize("pin", ORDER_FREE_GENERAL, ids=lambda p: p.__name__)
def test_pins_of_the_transposed_signature_through_strides_on_the_device(gpu_device, pin, c_layout, dtype):
    with pins.precision(dtype):
        pin(ps.as_general_impl(device_call, c_layout))


def _scale(alpha, A, B, beta, C0):
    # A, B, C0 are the logical operands (dense, row-major), so the scale of the strided operation is that of the
    # plain signature: the routine pinned by tests/test_oracle_scale_pins.py
    return oracle.general_scale(0, 0, alpha, A, B, beta, C0)


def _operands(seed, M, N, K, kind, dtype):
    rng = np.random.default_rng(seed)
    if kind == "int":
        gen = lambda r, c: rng.integers(-4, 5, size=(r, c)).astype(dtype)
    else:
        gen = lambda r, c: rng.uniform(-1, 1, size=(r, c)).astype(dtype)
    return gen(M, K), gen(K, N), gen(M, N)


def _check(alpha, A, B, beta, C0, layouts, kind, what):
    la, lb, lc = layouts
    with pins.precision(C0.dtype.type):
        Ab, Av = ps.place(A, la)
        Bb, Bv = ps.place(B, lb)
        Cb, Cv = ps.place(C0, lc)
        want_b, want = ps.place(C0, lc)
    oracle.gemm_strided_ref(alpha, Av, Bv, beta, want)
    device_call(alpha, Av, Bv, beta, Cv)
    assert ps.untouched(Cb, Cv), what + ": memory between the elements of C changed"
    got = np.ascontiguousarray(Cv)
    if kind == "int":
        pins.assert_bitwise(got, np.ascontiguousarray(want), what)
    else:
        gpu_util.check_tolerance(got, np.ascontiguousarray(want), _scale(alpha, A, B, beta, C0), what)


UNIT = ["row", "col"]
SHAPES = [(65, 63, 17), (129, 127, 31), (200, 264, 150), (257, 130, 65), (96, 400, 129)]


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("kind", ["int", "uniform"])
def test_unit_stride_layouts_over_several_tiles(gpu_device, kind, dtype):
    # row-major and column-major in every combination: all of them run on the tiled kernels
    t = 0
    for (M, N, K) in SHAPES:
        A, B, C0 = _operands(100 + t, M, N, K, kind, dtype)
        for la in UNIT:
            for lb in UNIT:
                for lc in UNIT:
                    alpha, beta = [(1.0, 1.0), (-1.5, 0.5), (2.0, 0.0), (0.25, -1.25)][t % 4]
                    t += 1
                    _check(alpha, A, B, beta, C0, (la, lb, lc), kind, "%s %s %s alpha %g beta %g" % ((M, N, K), (la, lb, lc), kind, alpha, beta))


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("kind", ["int", "uniform"])
def test_sampled_layouts(gpu_device, kind, dtype):
    # operands without a unit stride run on the tiled kernel's sampled mode: A and B gathered into the staging
    # buffers, C scattered
    t = 0
    for (M, N, K) in [(70, 50, 90), (33, 129, 64), (150, 7, 40), (200, 264, 150)]:
        A, B, C0 = _operands(200 + t, M, N, K, kind, dtype)
        for trip in [("row_step2", "row", "row"), ("row", "col_step3", "col"), ("col", "row", "row_step2"),
                     ("col_step3", "row_step2", "col_step3"), ("row", "row", "col_step3"), ("col_step3", "row_step2", "row"),
                     ("row_step2", "col_step3", "col"), ("col", "row_step2", "col")]:
            alpha, beta = [(1.0, 1.0), (-1.5, 0.5), (2.0, 0.0)][t % 3]
            t += 1
            _check(alpha, A, B, beta, C0, trip, kind, "%s %s %s" % ((M, N, K), trip, kind))


def test_the_path_rule_agrees_with_what_the_tests_above_assume():
    assert binding.gemm_f64_strided_path(70, 50, 90, 2 * 90 + 5, 2, 52, 1, 52, 1)[0] == 2       # row_step2, row, row
    assert binding.gemm_f64_strided_path(70, 50, 90, 92, 1, 52, 1, 2 * 50 + 5, 2)[0] == 2       # row, row, row_step2
    assert binding.gemm_f64_strided_path(70, 50, 90, 92, 1, 1, 93, 1, 73)[0] == 1               # row, col, col


def test_overlapping_read_only_operands_run_on_the_tiled_kernels(gpu_device):
    # A(i, k) = v[i + k] (strides 1, 1) and B(k, j) = w[2 k + j] (strides 2, 1) over several tiles
    M, N, K = 150, 140, 170
    rng = np.random.default_rng(9)
    v = rng.integers(-4, 5, size=M + K).astype(np.float64)
    w = rng.integers(-4, 5, size=2 * K + N).astype(np.float64)
    Av = np.lib.stride_tricks.as_strided(v, shape=(M, K), strides=(8, 8))
    Bv = np.lib.stride_tricks.as_strided(w, shape=(K, N), strides=(16, 8))
    assert binding.gemm_f64_strided_path(M, N, K, 1, 1, 2, 1, N, 1)[0] == 2
    C = np.zeros((M, N))
    device_call(1.0, Av, Bv, 0.0, C)
    want = np.zeros((M, N))
    oracle.gemm_strided_ref(1.0, Av, Bv, 0.0, want)
    pins.assert_bitwise(C, want, "Hankel operands")


def test_column_major_call_is_the_transposed_problem_bit_for_bit(gpu_device):
    # Fortran-style operands: everything column-major.  The library computes C^T = B^T A^T with the row-major
    # kernels, so the bits are those of that call through the transposed signature.
    M, N, K = 300, 520, 410
    A, B, C0 = _operands(7, M, N, K, "uniform", np.float64)
    Af, Bf, Cf = np.asfortranarray(A), np.asfortranarray(B), np.asfortranarray(C0)
    dA, dB, dC = (torch.from_numpy(x.T.copy()).to(DEV) for x in (Af, Bf, Cf))   # the stored (transposed) arrays
    dC2 = dC.clone()
    binding.gemm_f64_strided(M, N, K, 1.5, dA, 1, M, dB, 1, K, -0.5, dC, 1, M)
    binding.gemm_f64_general(0, 0, N, M, K, 1.5, dB, K, dA, M, -0.5, dC2, M)
    torch.cuda.synchronize()
    assert torch.equal(dC.view(torch.int64), dC2.view(torch.int64))
    want = C0.copy()
    oracle.gemm_strided_ref(1.5, A, B, -0.5, want)
    gpu_util.check_tolerance(dC.cpu().numpy().T, want, _scale(1.5, A, B, -0.5, C0), "column-major against the oracle")


def test_large_column_major_problem_matches_the_exact_integer_product(gpu_device):
    # full coverage at a size the oracle cannot do whole; sampled rows through the oracle
    M, N, K = 3001, 2500, 2049
    g = torch.Generator(device=DEV)
    g.manual_seed(3)
    A = torch.randint(-4, 5, (M, K), generator=g, device=DEV).double()
    B = torch.randint(-4, 5, (K, N), generator=g, device=DEV).double()
    C0 = torch.randint(-4, 5, (M, N), generator=g, device=DEV).double()
    lda, ldb, ldc = M + 3, K + 1, M + 2
    dA = torch.full((K, lda), float("nan"), dtype=torch.float64, device=DEV); dA[:, :M] = A.t()
    dB = torch.full((N, ldb), float("nan"), dtype=torch.float64, device=DEV); dB[:, :K] = B.t()
    dC = torch.full((N, ldc), float("nan"), dtype=torch.float64, device=DEV); dC[:, :M] = C0.t()
    binding.gemm_f64_strided(M, N, K, -2.0, dA, 1, lda, dB, 1, ldb, 1.0, dC, 1, ldc)
    torch.cuda.synchronize()
    assert torch.equal(dC[:, :M].t(), -2.0 * (A @ B) + C0)
    assert bool(torch.isnan(dC[:, M:]).all()), "padding of C written"
    rows = np.array([0, 1, 127, 128, 1500, 2999, 3000])
    want = np.ascontiguousarray(C0[rows].cpu().numpy())
    oracle.gemm_strided_ref(-2.0, np.ascontiguousarray(A[rows].cpu().numpy()), B.cpu().numpy(), 1.0, want)
    pins.assert_bitwise(dC[:, :M].t()[rows].cpu().numpy(), want, "oracle rows")


def test_seeded_random_layouts_match_the_exact_integer_product(gpu_device):
    # random shapes around the tile edges, random layouts per operand (padded, sampled, overlapping for A and B),
    # small integers: every correct evaluation is exact, so the product computed by the vendor library on gathered
    # copies is the answer (secondary to the oracle-based tests above); nothing outside C's elements may change
    rng = np.random.default_rng(2024)
    edges = [1, 2, 15, 16, 17, 31, 33, 63, 64, 65, 127, 129, 191, 193, 257]
    dim = lambda hi: int(rng.choice(edges)) if rng.random() < 0.5 else int(rng.integers(1, hi + 1))

    def layout(rows, cols, sampled_ok=True):
        kind, pad, s = int(rng.integers(6 if sampled_ok else 2)), int(rng.integers(0, 4)), int(rng.integers(2, 4))
        return [(cols + pad, 1), (1, rows + pad), (s * cols + pad, s), (s, s * rows + pad),
                (int(rng.integers(1, 4)), int(rng.integers(1, 4))), (s * (cols + pad), 1)][kind]

    span = lambda r, c, rs, cs: (max(r, 1) - 1) * rs + (max(c, 1) - 1) * cs + 1
    seen = {1: 0, 2: 0}
    sampled_c = 0
    for case in range(400):
        f32 = bool(rng.integers(2))
        dt, sz = (torch.float32, 4) if f32 else (torch.float64, 8)
        M, N, K = dim(300), dim(300), dim(400)
        alpha, beta = float(rng.choice([1, -1, 2, 0])), float(rng.choice([1, 0, -1, 2]))
        (rsa, csa), (rsb, csb) = layout(M, K), layout(K, N)
        rsc, csc = layout(M, N, sampled_ok=bool(rng.random() < 0.3))
        if M > 1 and N > 1 and not (rsc >= csc * (N - 1) + 1 or csc >= rsc * (M - 1) + 1):
            rsc, csc = N + 1, 1
        off = 5
        bufA = torch.randint(-3, 4, (off + span(M, K, rsa, csa) + 3,), device=DEV).to(dt)
        bufB = torch.randint(-3, 4, (off + span(K, N, rsb, csb) + 3,), device=DEV).to(dt)
        bufC = torch.full((off + span(M, N, rsc, csc) + 3,), float("nan"), dtype=dt, device=DEV)
        Av = torch.as_strided(bufA, (M, K), (rsa, csa), off)
        Bv = torch.as_strided(bufB, (K, N), (rsb, csb), off)
        Cv = torch.as_strided(bufC, (M, N), (rsc, csc), off)
        C0 = torch.randint(-3, 4, (M, N), device=DEV).to(dt)
        Cv.copy_(C0)
        want = alpha * (Av.double() @ Bv.double()) + (beta * C0.double() if beta != 0 else 0)
        a0, b0 = bufA.clone(), bufB.clone()
        path = binding.gemm_f64_strided_path(M, N, K, rsa, csa, rsb, csb, rsc, csc)
        seen[path[0]] += 1
        sampled_c += path[9] != 1
        fn = binding.gemm_f32_strided if f32 else binding.gemm_f64_strided
        fn(M, N, K, alpha, bufA.data_ptr() + off * sz, rsa, csa, bufB.data_ptr() + off * sz, rsb, csb, beta,
           bufC.data_ptr() + off * sz, rsc, csc)
        torch.cuda.synchronize()
        what = "case %d: f32=%d %s A%s B%s C%s alpha %g beta %g" % (case, f32, (M, N, K), (rsa, csa), (rsb, csb), (rsc, csc), alpha, beta)
        assert torch.equal(Cv.double(), want), what
        assert torch.equal(a0, bufA) and torch.equal(b0, bufB), what + ": A or B written"
        mask = torch.zeros_like(bufC, dtype=torch.bool)
        torch.as_strided(mask, (M, N), (rsc, csc), off).fill_(True)
        assert bool(torch.isnan(bufC[~mask]).all()), what + ": memory outside C's elements written"
    assert min(seen.values()) >= 20 and sampled_c >= 20, (seen, sampled_c)
