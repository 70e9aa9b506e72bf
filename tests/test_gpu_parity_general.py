"""C <- alpha * op(A) op(B) + beta * C on the GPU against its CPU oracle, through the C ABI, in both
precisions (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2003_00532_amd import binding, synth

import gpu_util
import pins
import pins_general as pg

pytestmark = pytest.mark.gpu

MFMA_VARIANTS = [1, 2, 3, 4]
COMBOS = pg.COMBOS
DTYPES = [np.float64, np.float32]

# shapes the oracle finishes quickly that span several macro-tiles and ragged tails in M, N and K
SHAPES = [(1, 1, 1), (17, 15, 3), (64, 64, 32), (65, 63, 17), (129, 127, 31), (200, 264, 150), (257, 130, 33),
          (96, 400, 129), (385, 70, 64)]
SCALARS = [(1.0, 1.0), (-1.5, 0.5), (2.0, 0.0), (0.3, -1.25)]


def _fn(dtype):
    return binding.gemm_f32_general_ex if np.dtype(dtype) == np.float32 else binding.gemm_f64_general_ex


def run_general(ta, tb, alpha, Asb, Bsb, beta, Cb, M, N, K, variant=-1):
    """Stored, padded host buffers -> device -> general GEMM -> the three device buffers back as NumPy."""
    dA, dB, dC = (gpu_util.to_dev(x) for x in (Asb, Bsb, Cb))
    _fn(Cb.dtype)(ta, tb, M, N, K, alpha, dA, Asb.shape[1], dB, Bsb.shape[1], beta, dC, Cb.shape[1], variant=variant)
    torch.cuda.synchronize()
    return dA.cpu().numpy(), dB.cpu().numpy(), dC.cpu().numpy()


def make_impl(variant=-1):
    """Adapter with the impl(ta, tb, alpha, A, B, beta, C) signature of tests/pins_general.py."""
    def impl(ta, tb, alpha, A, B, beta, C):
        M, N = C.shape
        K = A.shape[0] if ta else A.shape[1]
        bufs = []
        for x in (A, B, C):
            sz = x.dtype.itemsize
            ld = x.strides[0] // sz if (x.shape[0] > 1 and x.size and x.strides[0] // sz >= x.shape[1]) else max(1, x.shape[1])
            b = synth.padded(x.shape[0], x.shape[1], max(1, ld), dtype=x.dtype)
            b[:, :x.shape[1]] = x
            bufs.append(b)
        a2, b2, c2 = run_general(ta, tb, alpha, bufs[0], bufs[1], beta, bufs[2], M, N, K, variant=variant)
        assert synth.padding_intact(a2, A.shape[1]) and synth.padding_intact(b2, B.shape[1]) and synth.padding_intact(c2, N), \
            "device padding was written"
        C[...] = c2[:, :N]
    return impl


def check_general(ta, tb, alpha, As, Bs, beta, C0, got, integer, what):
    want = C0.copy()
    oracle.gemm_general_ref(ta, tb, alpha, As, Bs, beta, want)
    if integer:
        pins.assert_bitwise(got, want, what)
        return 0.0
    S = oracle.general_scale(ta, tb, alpha, As, Bs, beta, C0)
    return gpu_util.check_tolerance(got, want, S, what)


ORDER_FREE = [pg.pin_general_tiny_exact, pg.pin_general_all_ones, pg.pin_general_one_hot, pg.pin_general_unread_operands,
              pg.pin_general_integer_exact, pg.pin_general_error_bound]


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("pin", ORDER_FREE, ids=lambda p: p.__name__)
def test_order_independent_general_pins_hold_on_device(gpu_device, pin, dtype):
    with pins.precision(dtype):
        pin(make_impl())


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("variant", MFMA_VARIANTS + [0])
def test_one_hot_and_unread_operands_per_variant(gpu_device, variant, dtype):
    with pins.precision(dtype):
        pg.pin_general_one_hot(make_impl(variant))
        pg.pin_general_unread_operands(make_impl(variant))
        pg.pin_general_tiny_exact(make_impl(variant), limit=2)


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("combo", COMBOS, ids=["nn", "nt", "tn", "tt"])
@pytest.mark.parametrize("variant", [-1, 0] + MFMA_VARIANTS)
def test_general_small_shapes_elementwise(gpu_device, variant, combo, dtype):
    ta, tb = combo
    with pins.precision(dtype):
        for n, (M, N, K) in enumerate(SHAPES):
            for kind in ("int", "uniform"):
                alpha, beta = SCALARS[(n + ta + 2 * tb) % len(SCALARS)]
                if kind == "int":
                    alpha, beta = float(round(2 * alpha)), float(round(2 * beta))
                # pads (0, 0, 0) and (8, 4, 2) keep every stored row 16-byte aligned, (3, 5, 1) does not
                for pad in ((0, 0, 0), (8, 4, 2), (3, 5, 1)):
                    A, B, C0 = pg._logical(300 + n, M, N, K, kind="int" if kind == "int" else "uniform")
                    Ab, As = pg.stored(A, ta, pad=pad[0])
                    Bb, Bs = pg.stored(B, tb, pad=pad[1])
                    Cb, _ = pg.stored(C0, 0, pad=pad[2])
                    a2, b2, c2 = run_general(ta, tb, alpha, Ab, Bb, beta, Cb, M, N, K, variant=variant)
                    what = "variant %d %s %s trans %s pad %s alpha %g beta %g" % (variant, kind, (M, N, K), combo, pad, alpha, beta)
                    assert synth.padding_intact(c2, N) and synth.padding_intact(a2, As.shape[1]) and \
                        synth.padding_intact(b2, Bs.shape[1]), what
                    check_general(ta, tb, alpha, As, Bs, beta, C0, c2[:, :N], kind == "int", what)


THIN = [(5, (0, 0)), (5, (0, 1)), (6, (0, 1)), (6, (1, 1))]   # 32-row tiles need A as given, 32-column tiles a transposed B


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("variant,combo", THIN, ids=lambda x: str(x))
def test_thin_tile_variants_elementwise(gpu_device, variant, combo, dtype):
    ta, tb = combo
    with pins.precision(dtype):
        for n, (M, N, K) in enumerate(SHAPES + [(31, 33, 40), (95, 97, 200)]):
            for kind in ("int", "uniform"):
                alpha, beta = SCALARS[(n + variant) % len(SCALARS)]
                if kind == "int":
                    alpha, beta = float(round(2 * alpha)), float(round(2 * beta))
                for pad in ((0, 0, 0), (8, 4, 2), (3, 5, 1)):
                    A, B, C0 = pg._logical(400 + n, M, N, K, kind="int" if kind == "int" else "uniform")
                    Ab, As = pg.stored(A, ta, pad=pad[0])
                    Bb, Bs = pg.stored(B, tb, pad=pad[1])
                    Cb, _ = pg.stored(C0, 0, pad=pad[2])
                    a2, b2, c2 = run_general(ta, tb, alpha, Ab, Bb, beta, Cb, M, N, K, variant=variant)
                    what = "thin variant %d %s %s trans %s pad %s" % (variant, kind, (M, N, K), combo, pad)
                    assert synth.padding_intact(c2, N) and synth.padding_intact(a2, As.shape[1]) and \
                        synth.padding_intact(b2, Bs.shape[1]), what
                    check_general(ta, tb, alpha, As, Bs, beta, C0, c2[:, :N], kind == "int", what)


def test_thin_tile_variants_are_refused_for_the_other_layouts(gpu_device):
    d = torch.zeros(64 * 64, dtype=torch.float64, device="cuda:0")
    for variant, bad in ((5, [(1, 0), (1, 1)]), (6, [(0, 0), (1, 0)])):
        for (ta, tb) in bad:
            assert binding.gemm_f64_general_raw(ta, tb, 64, 64, 64, 1.0, d, 64, d, 64, 1.0, d, 64, variant=variant) == -9


@pytest.mark.parametrize("variant", [5])
def test_thin_tiles_on_the_edge_config(gpu_device, variant):
    w = synth.WORKLOADS["c2_edge"]
    Ab, Bb, Cb = synth.workload_inputs(w, seed=1, integer=True)
    a2, b2, c2 = gpu_util.run_device(Ab, Bb, Cb, w.M, w.N, w.K, variant=variant)
    assert synth.padding_intact(c2, w.N)
    gpu_util.check_against_oracle(Ab[:, :w.K], Bb[:, :w.N], Cb[:, :w.N], c2[:, :w.N], True, "c2 variant %d" % variant)


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("combo", COMBOS[1:], ids=["nt", "tn", "tt"])
@pytest.mark.parametrize("variant", MFMA_VARIANTS)
def test_transposed_edges(gpu_device, variant, combo, dtype):
    # leading dimensions that are multiples of four elements: edge tiles in M and N are
    # handled by row redirection (k-contiguous operand) or by masked cells plus 4-byte tail copies
    # (the other kind), whichever operand they belong to; every remainder class is visited
    ta, tb = combo
    K = 96
    with pins.precision(dtype):
        for (M, N) in [(130, 129), (129, 130), (67, 131), (200, 143), (75, 144), (190, 145), (64, 191), (127, 255),
                       (128, 257), (65, 65), (1, 1), (16, 2), (33, 3), (3, 33)]:
            A, B, C0 = pg._logical(11, M, N, K, kind="int")
            Ab, As = pg.stored(A, ta, pad=(-A.T.shape[1] if ta else -K) % 4 + 4)
            Bb, Bs = pg.stored(B, tb, pad=(-K if tb else -N) % 4 + 4)
            Cb, _ = pg.stored(C0, 0, pad=3)
            assert Ab.shape[1] % 4 == 0 and Bb.shape[1] % 4 == 0
            a2, b2, c2 = run_general(ta, tb, -2.0, Ab, Bb, 1.0, Cb, M, N, K, variant=variant)
            what = "variant %d edge %s trans %s" % (variant, (M, N, K), combo)
            assert synth.padding_intact(c2, N) and synth.padding_intact(a2, As.shape[1]) and synth.padding_intact(b2, Bs.shape[1]), what
            check_general(ta, tb, -2.0, As, Bs, 1.0, C0, c2[:, :N], True, what)


def test_general_with_unit_scalars_is_the_plain_entry_point_bit_for_bit(gpu_device):
    w = synth.WORKLOADS["c2_edge"]
    Ab, Bb, Cb = synth.workload_inputs(w, seed=2)
    _, _, c_plain = gpu_util.run_device(Ab, Bb, Cb, w.M, w.N, w.K)
    _, _, c_general = run_general(0, 0, 1.0, Ab, Bb, 1.0, Cb, w.M, w.N, w.K)
    pins.assert_bitwise(c_general, c_plain, "general(1, 1) vs gemm_f64")


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("combo", COMBOS, ids=["nn", "nt", "tn", "tt"])
def test_general_2048_every_element(gpu_device, combo, dtype):
    # the paper-sized square problem in the automatic launch configuration, every element; the oracle is
    # given the same logical operands as contiguous arrays (a transposed copy is data movement only)
    ta, tb = combo
    M = N = K = 2048
    alpha, beta = -0.75, 1.5
    with pins.precision(dtype):
        for kind in ("int", "uniform"):
            A, B, C0 = pg._logical(0, M, N, K, kind=kind)
            al, be = (-3.0, 2.0) if kind == "int" else (alpha, beta)
            As = np.ascontiguousarray(A.T) if ta else A
            Bs = np.ascontiguousarray(B.T) if tb else B
            _, _, c2 = run_general(ta, tb, al, As, Bs, be, C0, M, N, K)
            want = C0.copy()
            oracle.gemm_general_ref(0, 0, al, A, B, be, want)
            what = "2048^3 %s trans %s" % (kind, combo)
            if kind == "int":
                pins.assert_bitwise(c2, want, what)
            else:
                S = oracle.general_scale(0, 0, al, A, B, be, C0)
                print(what, "worst |diff|/S = %.3g" % gpu_util.check_tolerance(c2, want, S, what))


@pytest.mark.parametrize("combo", COMBOS[1:], ids=["nt", "tn", "tt"])
def test_general_8192_sampled_rows(gpu_device, combo):
    # the benchmark size with transposed operands and beta = 0 over a NaN-filled C: complete sampled rows
    ta, tb = combo
    M = N = K = 8192
    w = synth.WORKLOADS["c3_8192"]
    Ab, Bb, _ = synth.workload_inputs(w, seed=0)
    A, B = Ab[:, :K], Bb[:, :N]
    dA = gpu_util.to_dev(A).t().contiguous() if ta else gpu_util.to_dev(A)
    dB = gpu_util.to_dev(B).t().contiguous() if tb else gpu_util.to_dev(B)
    dC = torch.full((M, N), float("nan"), dtype=torch.float64, device="cuda:0")
    binding.gemm_f64_general(ta, tb, M, N, K, 0.5, dA, 8192, dB, 8192, 0.0, dC, 8192)
    torch.cuda.synchronize()
    rows = synth.sample_rows(M, 96, seed=4)
    got = dC[torch.from_numpy(rows).to("cuda:0")].cpu().numpy()
    Ar = np.ascontiguousarray(A[rows, :])
    want = np.full((len(rows), N), np.nan)
    oracle.gemm_general_ref(0, 0, 0.5, Ar, B, 0.0, want)
    S = oracle.general_scale(0, 0, 0.5, Ar, B, 0.0, want)
    print("8192^3 trans %s worst |diff|/S = %.3g" % (combo, gpu_util.check_tolerance(got, want, S, "8192 %s" % (combo,))))


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
def test_seeded_random_cases_differential(gpu_device, dtype):
    # 160 seeded cases per precision: random shape (ragged in every dimension, including zero sizes), random
    # paddings (aligned and not), random transposes, scalars from a set that includes 0 and 1, and a random
    # kernel variant among those that exist for the layout; integer data, so the bar is bit-exactness
    rng = np.random.default_rng(20030532)
    n_variants = binding.gemm_f64_variant_count()
    scal = [0.0, 1.0, -1.0, 2.0, -3.0, 0.5]
    with pins.precision(dtype):
        for case in range(160):
            M, N = int(rng.integers(0, 200)), int(rng.integers(0, 200))
            K = int(rng.choice([0, 1, 3, 15, 16, 17, 31, 32, 33, 64, 100, int(rng.integers(1, 260))]))
            ta, tb = int(rng.integers(2)), int(rng.integers(2))
            alpha, beta = float(rng.choice(scal)), float(rng.choice(scal))
            pads = [int(rng.choice([0, 1, 2, 3, 4, 7, 8])) for _ in range(3)]
            variant = int(rng.integers(-1, n_variants))
            if (variant == 5 and ta) or (variant == 6 and not tb):
                variant = -1
            A, B, C0 = pg._logical(9000 + case, M, N, K, kind="int")
            Ab, As = pg.stored(A, ta, pad=pads[0])
            Bb, Bs = pg.stored(B, tb, pad=pads[1])
            Cb, _ = pg.stored(C0, 0, pad=pads[2])
            a2, b2, c2 = run_general(ta, tb, alpha, Ab, Bb, beta, Cb, M, N, K, variant=variant)
            what = "case %d: %s trans %s alpha %g beta %g pads %s variant %d" % (case, (M, N, K), (ta, tb), alpha, beta, pads, variant)
            assert synth.padding_intact(c2, N) and synth.padding_intact(a2, As.shape[1]) and synth.padding_intact(b2, Bs.shape[1]), what
            check_general(ta, tb, alpha, As, Bs, beta, C0, c2[:, :N], True, what)
