"""The two ways the double-precision kernels update C when alpha == beta == 1 (load-add-store by the lane, or additions
performed by the memory system) must give the same bits, special values included, and the automatic choice must fall
back to the first for memory that is not ordinary device memory (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2003_00532_amd import binding, synth

import gpu_util
import pins

pytestmark = pytest.mark.gpu
LOAD_STORE, IN_MEMORY = 1, 2


@pytest.fixture
def epilogue_mode():
    prev = binding.gemm_f64_set_epilogue_mode(0)
    yield binding.gemm_f64_set_epilogue_mode
    binding.gemm_f64_set_epilogue_mode(prev)


def _run(mode, set_mode, Ab, Bb, Cb, M, N, K, variant):
    set_mode(mode)
    try:
        return gpu_util.run_device(Ab, Bb, Cb, M, N, K, variant=variant)[2]
    finally:
        set_mode(0)


def _same_bits_or_both_nan(x, y, what):
    nan = np.isnan(x)
    assert np.array_equal(nan, np.isnan(y)), what + ": NaN in different places"
    bad = np.flatnonzero((x.view(np.uint64) != y.view(np.uint64)) & ~nan)
    assert bad.size == 0, "%s: %d elements differ (first flat index %d: %r vs %r)" % (what, bad.size, bad[0], x.ravel()[bad[0]], y.ravel()[bad[0]])


@pytest.mark.parametrize("variant", [-1, 1, 2, 3, 4, 5])
def test_both_forms_give_the_same_bits_on_uniform_data(gpu_device, epilogue_mode, variant):
    # ragged and full shapes, padded leading dimensions: every tile kind, edge predicates included
    for n, (M, N, K) in enumerate([(128, 128, 64), (129, 127, 31), (300, 275, 47), (256, 384, 512), (385, 70, 300)]):
        Ab, A = synth.matrix(40 + n, synth.TAG_A, M, K, K + 2, "uniform")
        Bb, B = synth.matrix(40 + n, synth.TAG_B, K, N, N + 4, "uniform")
        Cb, C0 = synth.matrix(40 + n, synth.TAG_C, M, N, N + 3, "uniform")
        c_ls = _run(LOAD_STORE, epilogue_mode, Ab, Bb, Cb, M, N, K, variant)
        c_im = _run(IN_MEMORY, epilogue_mode, Ab, Bb, Cb, M, N, K, variant)
        what = "variant %d %s" % (variant, (M, N, K))
        assert synth.padding_intact(c_im, N), what + ": padding written by the in-memory form"
        pins.assert_bitwise(c_im, c_ls, what)
        gpu_util.check_against_oracle(A, B, C0, c_im[:, :N], False, what)


def test_both_forms_agree_on_special_values(gpu_device, epilogue_mode):
    # C holds infinities, NaN, signed zeros, subnormals and the largest finite values; the sums include exact zeros
    # (zero rows of A), subnormal sums (tiny operands), overflowing sums and infinities
    M, N, K = 192, 160, 48
    rng = np.random.default_rng(3)
    A = rng.uniform(-1, 1, (M, K)); B = rng.uniform(-1, 1, (K, N))
    A[0:16, :] = 0.0                      # sums of +0 products: exact +0
    A[16:32, :] *= 2.0 ** -505; B[:, 0:40] *= 2.0 ** -505   # rows 16..31 x columns 0..39: sums around 2^-1010, next to the subnormal values of C
    A[32:48, :] *= 2.0 ** 600; B[:, 40:80] *= 2.0 ** 500    # overflow to infinity
    A[48, 3] = np.inf
    specials = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 5e-324, -5e-324, 2.0 ** -1040, -(2.0 ** -1040), 2.0 ** -1022,
                         np.finfo(np.float64).max, -np.finfo(np.float64).max, 1.0, -1.0, 2.0 ** -1080, 3.0 * 2.0 ** -1075])
    C0 = specials[rng.integers(0, len(specials), (M, N))]
    for variant in (-1, 1, 2, 4, 5):
        c_ls = _run(LOAD_STORE, epilogue_mode, A, B, C0.copy(), M, N, K, variant)
        c_im = _run(IN_MEMORY, epilogue_mode, A, B, C0.copy(), M, N, K, variant)
        _same_bits_or_both_nan(c_im, c_ls, "special values, variant %d" % variant)
        # rows of zeros in A leave C as it was (its subnormal values included: the addition does not flush them),
        # except that -0 + (+0) is +0
        want = C0[0:16].copy(); want[(want == 0)] = 0.0
        _same_bits_or_both_nan(np.ascontiguousarray(c_im[0:16]), want, "zero rows, variant %d" % variant)
        assert np.any((np.abs(want) > 0) & (np.abs(want) < 2.0 ** -1022)), "the zero rows were meant to meet subnormal values of C"


def test_automatic_choice_and_host_memory(gpu_device, epilogue_mode):
    # K >= 256 and 2^20 outputs: the automatic rule takes the in-memory form for device memory.  For C in page-locked
    # host memory mapped into the device it must not (such additions are not defined there), also when forced.
    M = N = 1024
    K = 256
    Ab, Bb, Cb = (synth.matrix(5, t, r, c, None, "int")[0] for t, r, c in ((synth.TAG_A, M, K), (synth.TAG_B, K, N), (synth.TAG_C, M, N)))
    want = Cb.copy()
    oracle.gemm_f64_ref(Ab, Bb, want)
    dA, dB = gpu_util.to_dev(Ab), gpu_util.to_dev(Bb)
    for mode in (0, IN_MEMORY, LOAD_STORE):
        epilogue_mode(mode)
        dC = gpu_util.to_dev(Cb)
        binding.gemm_f64(M, N, K, dA, K, dB, N, dC, N)
        torch.cuda.synchronize()
        pins.assert_bitwise(dC.cpu().numpy(), want, "device C, mode %d" % mode)
        hC = torch.empty((M, N), dtype=torch.float64, pin_memory=True)
        hC.copy_(torch.from_numpy(Cb))
        binding.gemm_f64(M, N, K, dA, K, dB, N, hC.data_ptr(), N)
        torch.cuda.synchronize()
        pins.assert_bitwise(hC.numpy(), want, "page-locked host C, mode %d" % mode)
    epilogue_mode(0)
    with pytest.raises(binding.GemmF64Error):
        binding.gemm_f64_set_epilogue_mode(7)


def test_in_memory_form_under_graph_capture(gpu_device, epilogue_mode):
    # the automatic rule asks the runtime who owns C; that query, and the additions in memory, must work in a captured
    # stream and on every replay
    M = N = 1024
    K = 256
    Ab, Bb, Cb = (synth.matrix(6, t, r, c, None, "int")[0] for t, r, c in ((synth.TAG_A, M, K), (synth.TAG_B, K, N), (synth.TAG_C, M, N)))
    want = Cb.copy()
    oracle.gemm_f64_ref(Ab, Bb, want)
    dA, dB, c_init = gpu_util.to_dev(Ab), gpu_util.to_dev(Bb), gpu_util.to_dev(Cb)
    out = torch.empty_like(c_init)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            out.copy_(c_init)
            binding.gemm_f64(M, N, K, dA, K, dB, N, out, N, stream=side)
    for rep in range(3):
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        pins.assert_bitwise(out.cpu().numpy(), want, "graph replay %d" % rep)
        _ = (dA[:8, :8] @ dB[:8, :8]).sum().item()


def test_products_below_the_normal_range(gpu_device):
    # Sums of products that are themselves subnormal (operands around 2^-540): the CPU definition keeps them as
    # subnormal numbers; the matrix unit is allowed to return them as they are or as signed zeros (it flushes them on
    # MI355X).  Either way nothing else may change, and sums in the normal range next to them are unaffected.
    M, N, K = 64, 64, 32
    rng = np.random.default_rng(8)
    A = rng.uniform(0.5, 1.0, (M, K)); B = rng.uniform(0.5, 1.0, (K, N)); C0 = np.zeros((M, N))
    A[:32] *= 2.0 ** -540; B[:, :32] *= 2.0 ** -540       # top-left quadrant: sums around 2^-1076
    _, _, got = gpu_util.run_device(A, B, C0.copy(), M, N, K)
    want = C0.copy(); oracle.gemm_f64_ref(A, B, want)
    tiny = got[:32, :32]
    flushed = bool(np.all(tiny == 0))
    kept = bool(np.all(np.abs(tiny - want[:32, :32]) <= 2.0 ** -1074 * K))
    print("subnormal products: %s" % ("flushed to zero" if flushed else "kept" if kept else "mixed"))
    assert flushed or kept
    S = np.zeros((M, N)); oracle.gemm_f64_absref(A, B, S)
    rest = np.ones((M, N), bool); rest[:32, :32] = False
    assert np.all(np.abs(got - want)[rest] <= 1e-13 * S[rest])


def test_fine_grained_device_memory(gpu_device, epilogue_mode):
    # C in device memory allocated fine-grained (coherent with the host at a finer grain): still device memory to the
    # runtime's query, and the additions in memory are performed there as in ordinary device memory
    import ctypes
    try:
        hip = ctypes.CDLL("libamdhip64.so")
        alloc, free, copy = hip.hipExtMallocWithFlags, hip.hipFree, hip.hipMemcpy
    except (OSError, AttributeError):
        pytest.skip("HIP runtime entry points not reachable through ctypes")
    M = N = 1024
    K = 256
    Ab, Bb, Cb = (synth.matrix(7, t, r, c, None, "int")[0] for t, r, c in ((synth.TAG_A, M, K), (synth.TAG_B, K, N), (synth.TAG_C, M, N)))
    want = Cb.copy()
    oracle.gemm_f64_ref(Ab, Bb, want)
    dA, dB = gpu_util.to_dev(Ab), gpu_util.to_dev(Bb)
    p = ctypes.c_void_p()
    if alloc(ctypes.byref(p), ctypes.c_size_t(M * N * 8), ctypes.c_uint(1)) != 0 or not p.value:   # hipDeviceMallocFinegrained
        pytest.skip("fine-grained device memory not available")
    try:
        for mode in (0, IN_MEMORY, LOAD_STORE):
            assert copy(p, ctypes.c_void_p(Cb.ctypes.data), ctypes.c_size_t(M * N * 8), 1) == 0
            epilogue_mode(mode)
            binding.gemm_f64(M, N, K, dA, K, dB, N, p.value, N)
            torch.cuda.synchronize()
            out = np.empty((M, N))
            assert copy(ctypes.c_void_p(out.ctypes.data), p, ctypes.c_size_t(M * N * 8), 2) == 0
            pins.assert_bitwise(out, want, "fine-grained C, mode %d" % mode)
    finally:
        epilogue_mode(0)
        free(p)
