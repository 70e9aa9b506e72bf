"""Single-precision HIP path against the float32 CPU oracle, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2003_00532_amd import binding, synth

import gpu_util
import pins

pytestmark = pytest.mark.gpu
F32 = np.float32
MFMA_VARIANTS = [1, 2, 3, 4]
ALL_VARIANTS = [-1, 0, 1, 2, 3, 4]

# several macro-tiles, ragged tails in M, N and K (K below, at and above one 32-deep stage, tails that
# are not multiples of the 4-element cell)
SHAPES = [
    (1, 1, 1), (16, 16, 4), (17, 15, 3), (64, 64, 32), (65, 63, 33), (128, 128, 64),
    (129, 127, 31), (200, 264, 150), (257, 130, 65), (300, 275, 47), (96, 400, 129), (385, 70, 96),
]


@pytest.fixture(autouse=True)
def _single_precision():
    with pins.precision(F32):
        yield


def _case(M, N, K, pad, kind, seed):
    lda, ldb, ldc = max(1, K + pad[0]), max(1, N + pad[1]), max(1, N + pad[2])
    Ab, A = synth.matrix(seed, synth.TAG_A, M, K, lda, kind, F32)
    Bb, B = synth.matrix(seed, synth.TAG_B, K, N, ldb, kind, F32)
    Cb, C = synth.matrix(seed, synth.TAG_C, M, N, ldc, kind, F32)
    return Ab, A, Bb, B, Cb, C


@pytest.mark.parametrize("variant", ALL_VARIANTS)
@pytest.mark.parametrize("kind", ["int", "uniform"])
def test_small_shapes_elementwise(gpu_device, variant, kind):
    for n, (M, N, K) in enumerate(SHAPES):
        # paddings that make ld a multiple of 4 keep rows 16-byte aligned for some shapes; for the others rows
        # start 4, 8 or 12 bytes off, which the 16-byte global->LDS copies must cope with
        for pad in ((0, 0, 0), ((-K) % 4 + 4, (-N) % 4 + 8, 2), (3, 5, 1)):
            Ab, A, Bb, B, Cb, C = _case(M, N, K, pad, kind, 100 + n)
            a2, b2, c2 = gpu_util.run_device(Ab, Bb, Cb, M, N, K, variant=variant)
            what = "f32 variant %d %s %s pad %s" % (variant, kind, (M, N, K), pad)
            assert synth.padding_intact(c2, N) and synth.padding_intact(a2, K) and synth.padding_intact(b2, N), what
            gpu_util.check_against_oracle(A, B, C, c2[:, :N], kind == "int", what)


@pytest.mark.parametrize("variant", MFMA_VARIANTS)
def test_right_and_bottom_edges_on_the_async_path(gpu_device, variant):
    # aligned operands with ld multiples of 4: every remainder of N modulo the 4-element cell and around
    # the 16-column MFMA tiles and the macro-tile, bottom edges too
    K = 96
    for (M, N) in [(130, 129), (129, 130), (67, 131), (200, 143), (75, 144), (190, 145), (64, 190), (127, 255),
                   (128, 257), (65, 65), (1, 1), (16, 2), (33, 3), (40, 66), (70, 67)]:
        lda, ldb, ldc = K + 4, N + (-N) % 4 + 4, N + 3
        Ab, A = synth.matrix(11, synth.TAG_A, M, K, lda, "int", F32)
        Bb, B = synth.matrix(11, synth.TAG_B, K, N, ldb, "int", F32)
        Cb, C = synth.matrix(11, synth.TAG_C, M, N, ldc, "int", F32)
        a2, b2, c2 = gpu_util.run_device(Ab, Bb, Cb, M, N, K, variant=variant)
        what = "f32 variant %d edge %s" % (variant, (M, N, K))
        assert synth.padding_intact(c2, N) and synth.padding_intact(a2, K) and synth.padding_intact(b2, N), what
        gpu_util.check_against_oracle(A, B, C, c2[:, :N], True, what)


@pytest.mark.parametrize("variant", [-1, 1, 2])
def test_misaligned_base_pointers(gpu_device, variant):
    M, N, K = 150, 140, 72
    for kind in ("int", "uniform"):
        Ab, A, Bb, B, Cb, C = _case(M, N, K, (4, 4, 4), kind, 7)
        lda, ldb, ldc = Ab.shape[1], Bb.shape[1], Cb.shape[1]
        flat = [torch.full((x.size + 1,), float("nan"), dtype=torch.float32, device="cuda:0") for x in (Ab, Bb, Cb)]
        for f, x in zip(flat, (Ab, Bb, Cb)):
            f[1:] = torch.from_numpy(x.ravel()).to("cuda:0")
        ptrs = [f.data_ptr() + 4 for f in flat]
        assert all(p % 16 == 4 for p in ptrs)
        binding.gemm_f32_ex(M, N, K, ptrs[0], lda, ptrs[1], ldb, ptrs[2], ldc, variant=variant)
        torch.cuda.synchronize()
        c2 = flat[2][1:].cpu().numpy().reshape(M, ldc)
        assert synth.padding_intact(c2, N)
        gpu_util.check_against_oracle(A, B, C, c2[:, :N], kind == "int", "f32 misaligned %s" % kind)


ORDER_FREE_PINS = [pins.pin_all_ones_small, pins.pin_identity, pins.pin_column_sums, pins.pin_rank_one,
                   pins.pin_one_hot_index, pins.pin_tiny_exact, pins.pin_integer_exact,
                   pins.pin_error_bound, pins.pin_ld_independence, pins.pin_degenerate]


@pytest.mark.parametrize("pin", ORDER_FREE_PINS, ids=lambda p: p.__name__)
def test_order_independent_pins_hold_on_device(gpu_device, pin):
    pin(gpu_util.make_impl())


@pytest.mark.parametrize("variant", MFMA_VARIANTS)
def test_one_hot_and_tiny_exact_per_variant(gpu_device, variant):
    # one-hot operands expose any error in the MFMA lane layout (which differs from the double one in
    # the result registers) or in the LDS cell layout
    pins.pin_one_hot_index(gpu_util.make_impl(variant))
    pins.pin_tiny_exact(gpu_util.make_impl(variant), limit=3)
    pins.pin_identity(gpu_util.make_impl(variant))


def test_block_split_invariance_on_device(gpu_device):
    pins.pin_block_split_invariance(gpu_util.make_impl(), bitwise_k=False)


@pytest.mark.parametrize("name", ["c0_256", "c1_2048", "c2_edge"])
@pytest.mark.parametrize("integer", [True, False], ids=["int", "uniform"])
def test_full_configs_against_oracle(gpu_device, name, integer):
    w = synth.WORKLOADS[name]
    Ab, Bb, Cb = synth.workload_inputs(w, seed=0, integer=integer, dtype=F32)
    a2, b2, c2 = gpu_util.run_device(Ab, Bb, Cb, w.M, w.N, w.K)
    assert synth.padding_intact(c2, w.N) and synth.padding_intact(a2, w.K) and synth.padding_intact(b2, w.N)
    ratio = gpu_util.check_against_oracle(Ab[:, :w.K], Bb[:, :w.N], Cb[:, :w.N], c2[:, :w.N], integer, name)
    print("f32 %s %s worst |diff|/S = %.3g (u = %.3g)" % (name, "int" if integer else "uniform", ratio, 2.0 ** -24))


@pytest.mark.parametrize("name,nrows", [("c3_8192", 192), ("c4_rankk", 1024)])
@pytest.mark.parametrize("integer", [True, False], ids=["int", "uniform"])
def test_large_configs_sampled_rows(gpu_device, name, nrows, integer):
    w = synth.WORKLOADS[name]
    Ab, Bb, Cb = synth.workload_inputs(w, seed=0, integer=integer, dtype=F32)
    dA, dB, dC = (gpu_util.to_dev(x) for x in (Ab, Bb, Cb))
    binding.gemm_f32(w.M, w.N, w.K, dA, w.lda, dB, w.ldb, dC, w.ldc)
    torch.cuda.synchronize()
    rows = synth.sample_rows(w.M, nrows, seed=3)
    got = dC[torch.from_numpy(rows).to("cuda:0")].cpu().numpy()[:, :w.N]
    A, B, C0 = Ab[:, :w.K], Bb[:, :w.N], Cb[:, :w.N]
    want = oracle.ref_rows(A, B, C0, rows)
    if integer:
        pins.assert_bitwise(got, want, name + " sampled rows")
    else:
        S = oracle.abs_rows(A, B, rows)
        ratio = gpu_util.check_tolerance(got, want, S, name + " sampled rows")
        print("f32 %s worst |diff|/S on %d rows = %.3g (u = %.3g)" % (name, len(rows), ratio, 2.0 ** -24))


@pytest.mark.parametrize("name", ["c4_rankk", "c3_8192"])
@pytest.mark.parametrize("integer", [True, False], ids=["int", "uniform"])
def test_large_configs_full_result(gpu_device, name, integer):
    # every element of the two largest configurations against the oracle, in the launch configuration the
    # benchmark times (automatic variant): bit-exact on integer data, within the tolerance on uniform data.
    # The inputs are generated on the device (the same bits as the host generator, see test_device_generator_*)
    # and copied to the host for the oracle.
    w = synth.WORKLOADS[name]
    dA, dB, dC = synth.device_workload_inputs(w, seed=0, integer=integer, dtype=F32)
    Ab, Bb, Cb = (x.cpu().numpy() for x in (dA, dB, dC))
    binding.gemm_f32(w.M, w.N, w.K, dA, w.lda, dB, w.ldb, dC, w.ldc)
    torch.cuda.synchronize()
    c2 = dC.cpu().numpy()
    del dA, dB, dC
    assert synth.padding_intact(c2, w.N)
    ratio = gpu_util.check_full_in_row_blocks(Ab[:, :w.K], Bb[:, :w.N], Cb[:, :w.N], c2[:, :w.N], integer, "f32 " + name)
    print("f32 %s %s full result: worst |diff|/S = %.3g (u = %.3g)" % (name, "int" if integer else "uniform", ratio, 2.0 ** -24))


@pytest.mark.parametrize("name", ["c3_8192", "c4_rankk"])
def test_large_configs_all_ones_everywhere(gpu_device, name):
    w = synth.WORKLOADS[name]
    dA = torch.ones((w.M, w.lda), dtype=torch.float32, device="cuda:0")
    dB = torch.ones((w.K, w.ldb), dtype=torch.float32, device="cuda:0")
    dC = torch.ones((w.M, w.ldc), dtype=torch.float32, device="cuda:0")
    binding.gemm_f32(w.M, w.N, w.K, dA, w.lda, dB, w.ldb, dC, w.ldc)
    torch.cuda.synchronize()
    assert bool(torch.all(dC[:, :w.N] == float(1 + w.K)))


def test_nonfinite_does_not_meet_k_padding(gpu_device):
    M, N, K = 20, 18, 5
    A = np.ones((M, K), F32); B = np.ones((K, N), F32); C = np.zeros((M, N), F32)
    A[3, 4] = np.inf
    B[2, 7] = np.inf
    _, _, c2 = gpu_util.run_device(A, B, C, M, N, K)
    want = np.full((M, N), float(K), F32); want[3, :] = np.inf; want[:, 7] = np.inf
    pins.assert_bitwise(c2, want, "Inf propagation")
