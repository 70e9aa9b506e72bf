"""HIP path against the CPU oracle, element by element, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2003_00532_amd import binding, synth

import gpu_util
import pins

pytestmark = pytest.mark.gpu

MFMA_VARIANTS = [1, 2, 3, 4]
ALL_VARIANTS = [-1, 0, 1, 2, 3, 4]

# sizes the oracle finishes in well under a second that still span several macro-tiles and ragged
# tails in M, N and K (K tails shorter and longer than one MFMA k-step, K below one LDS stage)
SHAPES = [
    (1, 1, 1), (16, 16, 4), (17, 15, 3), (64, 64, 16), (65, 63, 17), (128, 128, 32),
    (129, 127, 31), (200, 264, 150), (257, 130, 33), (300, 275, 47), (96, 400, 129), (385, 70, 64),
]


def _case(M, N, K, pad, kind, seed):
    lda, ldb, ldc = K + pad[0], N + pad[1], N + pad[2]
    Ab, A = synth.matrix(seed, synth.TAG_A, M, K, max(1, lda), kind)
    Bb, B = synth.matrix(seed, synth.TAG_B, K, N, max(1, ldb), kind)
    Cb, C = synth.matrix(seed, synth.TAG_C, M, N, max(1, ldc), kind)
    return Ab, A, Bb, B, Cb, C


@pytest.mark.parametrize("variant", ALL_VARIANTS)
@pytest.mark.parametrize("kind", ["int", "uniform"])
def test_small_shapes_elementwise(gpu_device, variant, kind):
    for n, (M, N, K) in enumerate(SHAPES):
        # even paddings keep rows 16-byte aligned, odd ones make every other row start 8 bytes off: the
        # 16-byte global->LDS copies must cope with both
        for pad in ((0, 0, 0), (8, 6, 2), (3, 5, 1)):
            Ab, A, Bb, B, Cb, C = _case(M, N, K, pad, kind, 100 + n)
            a2, b2, c2 = gpu_util.run_device(Ab, Bb, Cb, M, N, K, variant=variant)
            what = "variant %d %s %s pad %s" % (variant, kind, (M, N, K), pad)
            assert synth.padding_intact(c2, N) and synth.padding_intact(a2, K) and synth.padding_intact(b2, N), what
            gpu_util.check_against_oracle(A, B, C, c2[:, :N], kind == "int", what)


@pytest.mark.parametrize("variant", [-1, 1, 2])
def test_misaligned_base_pointers(gpu_device, variant):
    # bases 8 bytes off a 16-byte boundary: the 16-byte copies only need element alignment
    M, N, K = 150, 140, 70
    for kind in ("int", "uniform"):
        Ab, A, Bb, B, Cb, C = _case(M, N, K, (2, 2, 2), kind, 7)
        lda, ldb, ldc = Ab.shape[1], Bb.shape[1], Cb.shape[1]
        flat = [torch.full((x.size + 1,), float("nan"), dtype=torch.float64, device="cuda:0") for x in (Ab, Bb, Cb)]
        for f, x in zip(flat, (Ab, Bb, Cb)):
            f[1:] = torch.from_numpy(x.ravel()).to("cuda:0")
        ptrs = [f.data_ptr() + 8 for f in flat]
        assert all(p % 16 == 8 for p in ptrs)
        binding.gemm_f64_ex(M, N, K, ptrs[0], lda, ptrs[1], ldb, ptrs[2], ldc, variant=variant)
        torch.cuda.synchronize()
        c2 = flat[2][1:].cpu().numpy().reshape(M, ldc)
        assert synth.padding_intact(c2, N)
        gpu_util.check_against_oracle(A, B, C, c2[:, :N], kind == "int", "misaligned %s" % kind)


@pytest.mark.parametrize("variant", MFMA_VARIANTS)
def test_right_and_bottom_edges_on_the_async_path(gpu_device, variant):
    # aligned operands with even leading dimensions keep edge tiles on the global->LDS path: rows below
    # the matrix are redirected, column pairs outside it are masked and an odd last column is copied
    # on its own.  Every remainder class that matters is visited: 1, 2, odd, even, 15..17, one short.
    K = 80
    for (M, N) in [(130, 129), (129, 130), (67, 131), (200, 143), (75, 144), (190, 145), (64, 191), (127, 255),
                   (128, 257), (65, 65), (1, 1), (16, 2), (33, 3)]:
        lda, ldb, ldc = K + 2, N + (N % 2) + 4, N + 3
        Ab, A = synth.matrix(11, synth.TAG_A, M, K, lda, "int")
        Bb, B = synth.matrix(11, synth.TAG_B, K, N, ldb, "int")
        Cb, C = synth.matrix(11, synth.TAG_C, M, N, ldc, "int")
        a2, b2, c2 = gpu_util.run_device(Ab, Bb, Cb, M, N, K, variant=variant)
        what = "variant %d edge %s" % (variant, (M, N, K))
        assert synth.padding_intact(c2, N) and synth.padding_intact(a2, K) and synth.padding_intact(b2, N), what
        gpu_util.check_against_oracle(A, B, C, c2[:, :N], True, what)


@pytest.mark.parametrize("variant", [-1, 1, 2, 5])
def test_huge_leading_dimension_uses_64_bit_addressing(gpu_device, variant):
    # lda >= 2^22 elements is beyond the 32-bit lane offsets of the asynchronous copies: the register-staged
    # mode of the kernel takes over; checked on several shapes inside one 2.2 GB buffer (ragged edges, K tail)
    ld_big = (1 << 22) + 3
    rows = 140
    bufA = torch.full((rows, ld_big), float("nan"), dtype=torch.float64, device="cuda:0")
    for n, (M, N, K) in enumerate([(140, 70, 100), (64, 64, 64), (65, 130, 33), (129, 31, 17)]):
        _, A = synth.matrix(50 + n, synth.TAG_A, M, K, None, "int")
        Bb, B = synth.matrix(50 + n, synth.TAG_B, K, N, N + 1, "int")
        Cb, C = synth.matrix(50 + n, synth.TAG_C, M, N, N + 3, "int")
        bufA[:M, :K] = torch.from_numpy(A).to("cuda:0")
        dB, dC = gpu_util.to_dev(Bb), gpu_util.to_dev(Cb)
        binding.gemm_f64_ex(M, N, K, bufA, ld_big, dB, N + 1, dC, N + 3, variant=variant)
        torch.cuda.synchronize()
        c2 = dC.cpu().numpy()
        assert synth.padding_intact(c2, N)
        gpu_util.check_against_oracle(A, B, C, c2[:, :N], True, "huge lda %s variant %d" % ((M, N, K), variant))
    # and a huge ldb (B rows far apart), A dense
    K, N, M = 24, 40, 50
    bufB = torch.full((K, ld_big), float("nan"), dtype=torch.float64, device="cuda:0")
    _, A = synth.matrix(60, synth.TAG_A, M, K, None, "uniform")
    _, B = synth.matrix(60, synth.TAG_B, K, N, None, "uniform")
    Cb, C = synth.matrix(60, synth.TAG_C, M, N, N, "uniform")
    bufB[:, :N] = torch.from_numpy(B).to("cuda:0")
    dA, dC = gpu_util.to_dev(A), gpu_util.to_dev(Cb)
    binding.gemm_f64_ex(M, N, K, dA, K, bufB, ld_big, dC, N, variant=variant)
    torch.cuda.synchronize()
    gpu_util.check_against_oracle(A, B, C, dC.cpu().numpy(), False, "huge ldb variant %d" % variant)


def test_stale_lds_bits_do_not_reach_valid_columns(gpu_device):
    # a run on NaN data leaves NaN bits in LDS; the next launch has masked column pairs whose LDS cells
    # keep whatever was there, which must only ever feed columns that are not stored
    M, N, K = 256, 256, 64
    nan = torch.full((M, K), float("nan"), dtype=torch.float64, device="cuda:0")
    out = torch.zeros((M, N), dtype=torch.float64, device="cuda:0")
    for v in MFMA_VARIANTS:
        binding.gemm_f64_ex(M, N, K, nan, K, nan[:K, :].contiguous().repeat(1, N // K), N, out, N, variant=v)
    torch.cuda.synchronize()
    M, N, K = 70, 67, 48
    Ab, A = synth.matrix(12, synth.TAG_A, M, K, K, "int")
    Bb, B = synth.matrix(12, synth.TAG_B, K, N, N + 1, "int")
    Cb, C = synth.matrix(12, synth.TAG_C, M, N, N + 1, "int")
    for v in MFMA_VARIANTS:
        _, _, c2 = gpu_util.run_device(Ab, Bb, Cb, M, N, K, variant=v)
        gpu_util.check_against_oracle(A, B, C, c2[:, :N], True, "after NaN run, variant %d" % v)


ORDER_FREE_PINS = [pins.pin_all_ones_small, pins.pin_identity, pins.pin_column_sums, pins.pin_rank_one,
                   pins.pin_one_hot_index, pins.pin_tiny_exact, pins.pin_integer_exact,
                   pins.pin_error_bound, pins.pin_ld_independence, pins.pin_degenerate]


@pytest.mark.parametrize("pin", ORDER_FREE_PINS, ids=lambda p: p.__name__)
def test_order_independent_pins_hold_on_device(gpu_device, pin):
    # the facts that do not depend on summation order must hold for the HIP path as they do for the oracle
    pin(gpu_util.make_impl())


@pytest.mark.parametrize("variant", MFMA_VARIANTS)
def test_one_hot_and_tiny_exact_per_variant(gpu_device, variant):
    # one-hot operands expose any error in the MFMA lane layout or the LDS transposition
    pins.pin_one_hot_index(gpu_util.make_impl(variant))
    pins.pin_tiny_exact(gpu_util.make_impl(variant), limit=3)
    pins.pin_identity(gpu_util.make_impl(variant))


def test_block_split_invariance_on_device(gpu_device):
    pins.pin_block_split_invariance(gpu_util.make_impl(), bitwise_k=False)


@pytest.mark.parametrize("dtype", [np.float64, np.float32], ids=["f64", "f32"])
def test_device_generator_gives_the_host_generator_s_bits(gpu_device, dtype):
    iv = np.uint32 if dtype == np.float32 else np.uint64
    w = synth.WORKLOADS["c2_edge"]
    for integer in (False, True):
        host = synth.workload_inputs(w, seed=4, integer=integer, dtype=dtype)
        dev = synth.device_workload_inputs(w, seed=4, integer=integer, dtype=dtype)
        for h, d in zip(host, dev):
            assert np.array_equal(h.view(iv), d.cpu().numpy().view(iv))


@pytest.mark.parametrize("name", ["c0_256", "c1_2048", "c2_edge"])
@pytest.mark.parametrize("integer", [True, False], ids=["int", "uniform"])
def test_full_configs_against_oracle(gpu_device, name, integer):
    # whole result, every element, in the launch configuration the benchmark uses (automatic variant)
    w = synth.WORKLOADS[name]
    Ab, Bb, Cb = synth.workload_inputs(w, seed=0, integer=integer)
    a2, b2, c2 = gpu_util.run_device(Ab, Bb, Cb, w.M, w.N, w.K)
    assert synth.padding_intact(c2, w.N) and synth.padding_intact(a2, w.K) and synth.padding_intact(b2, w.N)
    ratio = gpu_util.check_against_oracle(Ab[:, :w.K], Bb[:, :w.N], Cb[:, :w.N], c2[:, :w.N], integer, name)
    print("%s %s worst |diff|/S = %.3g" % (name, "int" if integer else "uniform", ratio))


@pytest.mark.parametrize("variant", MFMA_VARIANTS)
def test_edge_config_every_variant(gpu_device, variant):
    w = synth.WORKLOADS["c2_edge"]
    Ab, Bb, Cb = synth.workload_inputs(w, seed=1, integer=True)
    a2, b2, c2 = gpu_util.run_device(Ab, Bb, Cb, w.M, w.N, w.K, variant=variant)
    assert synth.padding_intact(c2, w.N)
    gpu_util.check_against_oracle(Ab[:, :w.K], Bb[:, :w.N], Cb[:, :w.N], c2[:, :w.N], True, "c2 variant %d" % variant)


@pytest.mark.parametrize("name,nrows", [("c3_8192", 192), ("c4_rankk", 1024)])
@pytest.mark.parametrize("integer", [True, False], ids=["int", "uniform"])
def test_large_configs_sampled_rows(gpu_device, name, nrows, integer):
    # fast pre-check of the full-result test below: the oracle computes complete sampled rows (tile-boundary rows
    # plus hashed random ones); the device result must match on every element of those rows
    w = synth.WORKLOADS[name]
    Ab, Bb, Cb = synth.workload_inputs(w, seed=0, integer=integer)
    dA, dB, dC = (gpu_util.to_dev(x) for x in (Ab, Bb, Cb))
    binding.gemm_f64(w.M, w.N, w.K, dA, w.lda, dB, w.ldb, dC, w.ldc)
    torch.cuda.synchronize()
    rows = synth.sample_rows(w.M, nrows, seed=3)
    got = dC[torch.from_numpy(rows).to("cuda:0")].cpu().numpy()[:, :w.N]
    A, B, C0 = Ab[:, :w.K], Bb[:, :w.N], Cb[:, :w.N]
    want = oracle.ref_rows(A, B, C0, rows)
    if integer:
        pins.assert_bitwise(got, want, name + " sampled rows")
        # secondary, full-coverage cross-check: on integer data every correct fp64 GEMM is exact, so
        # the library routine behind torch.matmul must agree bit for bit on all M*N elements
        ref = to_full = torch.from_numpy(Cb).to("cuda:0")[:, :w.N] + dA[:, :w.K] @ dB[:, :w.N]
        assert torch.equal(dC[:, :w.N], ref), name + ": differs from the exact integer product somewhere"
    else:
        S = oracle.abs_rows(A, B, rows)
        ratio = gpu_util.check_tolerance(got, want, S, name + " sampled rows")
        print("%s worst |diff|/S on %d rows = %.3g" % (name, len(rows), ratio))


@pytest.mark.parametrize("name", ["c4_rankk", "c3_8192"])
@pytest.mark.parametrize("integer", [True, False], ids=["int", "uniform"])
def test_large_configs_full_result(gpu_device, name, integer):
    # every element of the two largest configurations against the oracle, in the launch configuration the
    # benchmark times (automatic variant): bit-exact on integer data, within the tolerance on uniform data.
    # The inputs are generated on the device (the same bits as the host generator, see test_device_generator_*)
    # and copied to the host for the oracle.
    w = synth.WORKLOADS[name]
    dA, dB, dC = synth.device_workload_inputs(w, seed=0, integer=integer)
    Ab, Bb, Cb = (x.cpu().numpy() for x in (dA, dB, dC))
    binding.gemm_f64(w.M, w.N, w.K, dA, w.lda, dB, w.ldb, dC, w.ldc)
    torch.cuda.synchronize()
    c2 = dC.cpu().numpy()
    del dA, dB, dC
    assert synth.padding_intact(c2, w.N)
    ratio = gpu_util.check_full_in_row_blocks(Ab[:, :w.K], Bb[:, :w.N], Cb[:, :w.N], c2[:, :w.N], integer, name)
    print("%s %s full result: worst |diff|/S = %.3g" % (name, "int" if integer else "uniform", ratio))


@pytest.mark.parametrize("name", ["c3_8192", "c4_rankk"])
def test_large_configs_all_ones_everywhere(gpu_device, name):
    # the paper's own driver input (all matrices 1.0): every element of the result is exactly 1 + K
    w = synth.WORKLOADS[name]
    dA = torch.ones((w.M, w.lda), dtype=torch.float64, device="cuda:0")
    dB = torch.ones((w.K, w.ldb), dtype=torch.float64, device="cuda:0")
    dC = torch.ones((w.M, w.ldc), dtype=torch.float64, device="cuda:0")
    binding.gemm_f64(w.M, w.N, w.K, dA, w.lda, dB, w.ldb, dC, w.ldc)
    torch.cuda.synchronize()
    assert bool(torch.all(dC[:, :w.N] == float(1 + w.K)))


def test_paper_shape_all_ones(gpu_device):
    pins.pin_paper_all_ones(gpu_util.make_impl())


def test_repeatable_and_stream(gpu_device):
    w = synth.WORKLOADS["c2_edge"]
    Ab, Bb, Cb = synth.workload_inputs(w, seed=5)
    _, _, c_first = gpu_util.run_device(Ab, Bb, Cb, w.M, w.N, w.K)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        _, _, c_second = gpu_util.run_device(Ab, Bb, Cb, w.M, w.N, w.K, stream=s)
    pins.assert_bitwise(c_first, c_second, "two runs, two streams")


def test_degenerate_sizes_touch_nothing(gpu_device):
    Cb, C = synth.matrix(9, synth.TAG_C, 5, 7, 9, "uniform")
    dC = gpu_util.to_dev(Cb)
    dA = torch.zeros(64, dtype=torch.float64, device="cuda:0")
    binding.gemm_f64(5, 7, 0, dA, 1, dA, 7, dC, 9)
    binding.gemm_f64(0, 7, 3, dA, 3, dA, 7, dC, 9)
    binding.gemm_f64(5, 0, 3, dA, 3, dA, 1, dC, 9)
    torch.cuda.synchronize()
    pins.assert_bitwise(dC.cpu().numpy(), Cb, "degenerate calls")


def test_nonfinite_does_not_meet_k_padding(gpu_device):
    # K = 5 leaves 11 zero-filled k slots in the LDS stage; an Inf in live data must give Inf, not NaN
    M, N, K = 20, 18, 5
    A = np.ones((M, K)); B = np.ones((K, N)); C = np.zeros((M, N))
    A[3, 4] = np.inf
    B[2, 7] = np.inf
    _, _, c2 = gpu_util.run_device(A, B, C, M, N, K)
    want = np.full((M, N), float(K)); want[3, :] = np.inf; want[:, 7] = np.inf
    pins.assert_bitwise(c2, want, "Inf propagation")
