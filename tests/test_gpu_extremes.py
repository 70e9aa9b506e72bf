"""Edges of the index range and of the calling conventions, on the GPU: buffers beyond 4 GiB, extreme aspect
ratios, aliased operands, capture into a HIP graph, concurrent host threads (needs an MI355X)."""
import threading

import numpy as np
import pytest
import torch

import oracle
from paper_2003_00532_amd import binding, synth

import gpu_util
import pins

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _device_ints(seed, rows, cols, ld):
    """Integer-valued {-4..4} device matrix (rows, ld) from a seeded device generator, NaN in the padding."""
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    buf = torch.full((rows, ld), float("nan"), dtype=torch.float64, device=DEV)
    buf[:, :cols] = torch.randint(-4, 5, (rows, cols), generator=g, device=DEV).double()
    return buf


def test_c_larger_than_4_gib(gpu_device):
    # M * ldc * 8 bytes = 5.3 GB: row offsets of C exceed 2^32 bytes.  Complete sampled rows go through the
    # oracle; the whole result is cross-checked against the exact integer product computed on the device
    M, N, K = 40000, 16384, 64
    ldc = N + 8
    dA, dB, dC = _device_ints(1, M, K, K + 2), _device_ints(2, K, N, N), _device_ints(3, M, N, ldc)
    c0 = dC.clone()
    binding.gemm_f64(M, N, K, dA, K + 2, dB, N, dC, ldc)
    torch.cuda.synchronize()
    rows = synth.sample_rows(M, 64, seed=5)
    idx = torch.from_numpy(rows).to(DEV)
    A = dA[idx][:, :K].cpu().numpy()
    C0 = c0[idx][:, :N].cpu().numpy()
    want = np.ascontiguousarray(C0)
    oracle.gemm_f64_ref(np.ascontiguousarray(A), dB.cpu().numpy(), want)
    pins.assert_bitwise(dC[idx][:, :N].cpu().numpy(), want, "rows of a 5.3 GB C")
    assert torch.equal(dC[:, :N], c0[:, :N] + dA[:, :K] @ dB), "differs from the exact integer product somewhere"
    assert bool(torch.isnan(dC[:, N:]).all()), "C padding was written"


def test_c_with_more_than_2_to_the_32_elements(gpu_device):
    # 65600^2 = 4.3e9 elements (34 GB): element indices of C pass 2^32, and one block per 256 elements would be more
    # threads than a launch may have.  Data are small integers, so every result is exact: the whole of C is compared
    # with the exact integer product computed on the device a block of rows at a time, sampled rows with the oracle.
    free, _ = torch.cuda.mem_get_info()
    if free < 60 * 2 ** 30:
        pytest.skip("needs 60 GB of free device memory")
    M = N = 65600
    K = 8
    dA, dB = _device_ints(11, M, K, K), _device_ints(12, K, N, N)
    dC = torch.empty((M, N), dtype=torch.float64, device=DEV)
    cols = torch.arange(N, device=DEV)
    step = 4096

    def c_in(r0, r1):
        rows = torch.arange(r0, r1, device=DEV)
        return ((rows[:, None] + cols[None, :]) % 7 - 3).double()

    for r0 in range(0, M, step):
        dC[r0:r0 + step] = c_in(r0, min(M, r0 + step))
    # no product: C <- 2 C by the scaling kernel alone
    binding.gemm_f64_general(0, 0, M, N, K, 0.0, dA, K, dB, N, 2.0, dC, N)
    torch.cuda.synchronize()
    for r0 in range(0, M, step):
        assert torch.equal(dC[r0:r0 + step], 2.0 * c_in(r0, min(M, r0 + step))), "scaling differs in rows from %d" % r0
    # the paper's operation on top of it
    binding.gemm_f64(M, N, K, dA, K, dB, N, dC, N)
    torch.cuda.synchronize()
    for r0 in range(0, M, step):
        r1 = min(M, r0 + step)
        assert torch.equal(dC[r0:r1], 2.0 * c_in(r0, r1) + dA[r0:r1] @ dB), "product differs in rows from %d" % r0
    rows = synth.sample_rows(M, 16, seed=3)
    idx = torch.from_numpy(rows).to(DEV)
    want = np.ascontiguousarray((2.0 * ((rows[:, None] + np.arange(N)[None, :]) % 7 - 3)).astype(np.float64))
    oracle.gemm_f64_ref(np.ascontiguousarray(dA[idx].cpu().numpy()), dB.cpu().numpy(), want)
    pins.assert_bitwise(dC[idx].cpu().numpy(), want, "rows of a C of 4.3e9 elements")
    # the untiled kernel strides over the elements in the same way (a smaller K: one thread per element is slow)
    dC2 = dC[:, :].view(M, N)
    for r0 in range(0, M, step):
        dC2[r0:r0 + step] = c_in(r0, min(M, r0 + step))
    binding.gemm_f64_ex(M, N, 2, dA, K, dB, N, dC2, N, variant=0)
    torch.cuda.synchronize()
    for r0 in range(0, M, step):
        r1 = min(M, r0 + step)
        assert torch.equal(dC2[r0:r1], c_in(r0, r1) + dA[r0:r1, :2] @ dB[:2]), "untiled kernel differs in rows from %d" % r0


@pytest.mark.parametrize("shape", [(1, 300000, 70), (300000, 1, 70), (3, 5, 100003), (2, 70001, 2), (70001, 2, 2),
                                   (100000, 3, 7), (5, 33, 1)])
def test_extreme_aspect_ratios(gpu_device, shape):
    M, N, K = shape
    for kind in ("int", "uniform"):
        Ab, A = synth.matrix(21, synth.TAG_A, M, K, K + 1, kind)
        Bb, B = synth.matrix(21, synth.TAG_B, K, N, N + 2, kind)
        Cb, C = synth.matrix(21, synth.TAG_C, M, N, N + 1, kind)
        a2, b2, c2 = gpu_util.run_device(Ab, Bb, Cb, M, N, K)
        assert synth.padding_intact(c2, N) and synth.padding_intact(a2, K) and synth.padding_intact(b2, N)
        gpu_util.check_against_oracle(A, B, C, c2[:, :N], kind == "int", "shape %s %s" % (shape, kind))


def test_a_and_b_may_be_the_same_buffer(gpu_device):
    n = 200
    Xb, X = synth.matrix(31, synth.TAG_A, n, n, n + 2, "int")
    Cb, C = synth.matrix(31, synth.TAG_C, n, n, n, "int")
    dX, dC = gpu_util.to_dev(Xb), gpu_util.to_dev(Cb)
    binding.gemm_f64(n, n, n, dX, n + 2, dX, n + 2, dC, n)
    torch.cuda.synchronize()
    gpu_util.check_against_oracle(X, X, C, dC.cpu().numpy(), True, "A and B aliased")
    # and X^T X through the general entry point, still one buffer
    dC2 = gpu_util.to_dev(Cb)
    binding.gemm_f64_general(1, 0, n, n, n, 2.0, dX, n + 2, dX, n + 2, -1.0, dC2, n)
    torch.cuda.synchronize()
    want = C.copy()
    oracle.gemm_general_ref(1, 0, 2.0, X, X, -1.0, want)
    pins.assert_bitwise(dC2.cpu().numpy(), want, "X^T X aliased")


def test_calls_can_be_captured_in_a_graph_and_replayed(gpu_device):
    # the library allocates nothing and synchronises nothing, so its launches can be recorded; every replay
    # (with eager work and synchronisations in between) must reproduce the eager result bit for bit
    M, N, K = 300, 260, 190
    Ab, A = synth.matrix(41, synth.TAG_A, M, K, K + 1, "uniform")
    Bb, B = synth.matrix(41, synth.TAG_B, K, N, N + 3, "uniform")
    Cb, C = synth.matrix(41, synth.TAG_C, M, N, N, "uniform")
    dA, dB, c_init = gpu_util.to_dev(Ab), gpu_util.to_dev(Bb), gpu_util.to_dev(Cb)
    eager = c_init.clone()
    binding.gemm_f64(M, N, K, dA, K + 1, dB, N + 3, eager, N)
    binding.gemm_f64_general(0, 0, M, N, K, 0.5, dA, K + 1, dB, N + 3, 0.0, eager, N)   # overwrites: result is replay-independent
    torch.cuda.synchronize()
    out = torch.empty_like(c_init)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            binding.gemm_f64(M, N, K, dA, K + 1, dB, N + 3, out, N, stream=side)
            binding.gemm_f64_general(0, 0, M, N, K, 0.5, dA, K + 1, dB, N + 3, 0.0, out, N, stream=side)
    for rep in range(4):
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        pins.assert_bitwise(out.cpu().numpy(), eager.cpu().numpy(), "graph replay %d" % rep)
        _ = (dA[:8, :8] @ dB[:8, :8]).sum().item()   # unrelated eager work between replays
    S = oracle.general_scale(0, 0, 0.5, A, B, 0.0, C)
    want = C.copy()
    oracle.gemm_general_ref(0, 0, 0.5, A, B, 0.0, want)
    gpu_util.check_tolerance(out.cpu().numpy(), want, S, "graph result against the oracle")


def test_concurrent_host_threads_on_their_own_streams(gpu_device):
    # no global state: four host threads, each with its own stream and operands, all results correct
    shapes = [(257, 130, 77), (64, 300, 129), (190, 190, 64), (33, 65, 300)]
    results, errors = {}, []

    def work(i):
        try:
            torch.cuda.set_device(0)
            M, N, K = shapes[i]
            Ab, A = synth.matrix(70 + i, synth.TAG_A, M, K, K + 1, "int")
            Bb, B = synth.matrix(70 + i, synth.TAG_B, K, N, N + 1, "int")
            Cb, C = synth.matrix(70 + i, synth.TAG_C, M, N, N + 1, "int")
            s = torch.cuda.Stream()
            with torch.cuda.stream(s):
                dA, dB, dC = gpu_util.to_dev(Ab), gpu_util.to_dev(Bb), gpu_util.to_dev(Cb)
                for _ in range(20):
                    dC.copy_(torch.from_numpy(Cb), non_blocking=False)
                    binding.gemm_f64(M, N, K, dA, K + 1, dB, N + 1, dC, N + 1, stream=s)
                s.synchronize()
                results[i] = (A, B, C, dC.cpu().numpy()[:, :N])
        except Exception as e:  # pragma: no cover
            errors.append(e)

    threads = [threading.Thread(target=work, args=(i,)) for i in range(len(shapes))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for i, (A, B, C, got) in results.items():
        gpu_util.check_against_oracle(A, B, C, got, True, "thread %d" % i)


def test_mfma_probe_runs_and_validates_its_arguments(gpu_device):
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.full((512 * cus,), float("nan"), dtype=torch.float64, device=DEV)
    flops = binding.gemm_f64_mfma_probe(10, sink, sink.numel())
    torch.cuda.synchronize()
    assert flops == 2 * cus * 4 * 10 * 16 * 2048.0
    # every thread wrote a finite value: 4 result elements x 16 tiles, each 10 iterations x 4 k of a*b
    assert bool(torch.isfinite(sink).all()) and float(sink.min()) > 0
    assert load_raw().gemm_f64_mfma_probe(10, sink.data_ptr(), sink.numel() - 1, None, None) == -1
    assert load_raw().gemm_f64_mfma_probe(0, sink.data_ptr(), sink.numel(), None, None) == -1
    assert load_raw().gemm_f64_mfma_probe(10, None, sink.numel(), None, None) == -5


def test_device_peak_matches_the_published_figures_of_the_part(gpu_device):
    cus, khz, p64, p32 = binding.gemm_f64_device_peak()
    assert cus == torch.cuda.get_device_properties(0).multi_processor_count
    assert p32 == 2 * p64 and abs(p64 - cus * 128 * khz * 1e3 / 1e12) < 1e-9
    if cus == 256 and khz == 2400000:
        assert abs(p64 - 78.6) < 0.05 and abs(p32 - 157.3) < 0.05


def load_raw():
    return binding.load()


def test_large_ragged_shapes_match_the_exact_integer_product_everywhere(gpu_device):
    # sizes the CPU oracle cannot do whole: on integer data every correct GEMM is exact, so the product computed
    # on the device by the vendor library serves as a full-coverage cross-check (secondary: the oracle-based
    # tests are the bar); complete sampled rows still go through the oracle
    rng = np.random.default_rng(7)
    for case in range(10):
        M, N, K = (int(rng.integers(1500, 5000)) for _ in range(3))
        ta, tb = int(rng.integers(2)), int(rng.integers(2))
        alpha, beta = float(rng.choice([1.0, -2.0, 3.0])), float(rng.choice([0.0, 1.0, -1.0]))
        g = torch.Generator(device=DEV)
        g.manual_seed(1000 + case)
        A = torch.randint(-4, 5, (M, K), generator=g, device=DEV).double()
        B = torch.randint(-4, 5, (K, N), generator=g, device=DEV).double()
        C0 = torch.randint(-4, 5, (M, N), generator=g, device=DEV).double()
        lda, ldb, ldc = (M if ta else K) + int(rng.integers(0, 4)), (K if tb else N) + int(rng.integers(0, 4)), N + int(rng.integers(0, 4))
        dA = torch.full((K if ta else M, lda), float("nan"), dtype=torch.float64, device=DEV)
        dB = torch.full((N if tb else K, ldb), float("nan"), dtype=torch.float64, device=DEV)
        dC = torch.full((M, ldc), float("nan"), dtype=torch.float64, device=DEV)
        dA[:, :(M if ta else K)] = A.t() if ta else A
        dB[:, :(K if tb else N)] = B.t() if tb else B
        dC[:, :N] = C0
        binding.gemm_f64_general(ta, tb, M, N, K, alpha, dA, lda, dB, ldb, beta, dC, ldc)
        torch.cuda.synchronize()
        what = "case %d: %s trans %s alpha %g beta %g" % (case, (M, N, K), (ta, tb), alpha, beta)
        assert torch.equal(dC[:, :N], alpha * (A @ B) + beta * C0), what
        assert bool(torch.isnan(dC[:, N:]).all()), what + ": C padding written"
        rows = synth.sample_rows(M, 24, seed=case)
        Ar = np.ascontiguousarray(A[torch.from_numpy(rows).to(DEV)].cpu().numpy())
        want = np.ascontiguousarray(C0[torch.from_numpy(rows).to(DEV)].cpu().numpy())
        oracle.gemm_general_ref(0, 0, alpha, Ar, B.cpu().numpy(), beta, want)
        pins.assert_bitwise(dC[torch.from_numpy(rows).to(DEV)][:, :N].cpu().numpy(), want, what + " (oracle rows)")
