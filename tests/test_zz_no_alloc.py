"""gemm_f64_general_static, the entry point that allocates nothing (split K on the library's own fixed scratch
buffer), against gemm_f64_general_ws with a caller's workspace and against the CPU oracle (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2003_00532_amd import binding

import gpu_util
import pins
import pins_general as pg

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both_ways(ta, tb, alpha, beta, M, N, K, kind, seed, cus):
    """One problem through the workspace form and through the static form on separate copies of C; returns both
    results, the plan, and the operands (as stored, with their padded buffers)."""
    variant, splits, chunk = binding.gemm_f64_split_k_plan(ta, tb, M, N, K, cus)
    tail_tiles = binding.gemm_f64_tail_split_plan(ta, tb, M, N, K, cus)[1]
    ws_bytes = binding.gemm_f64_split_k_workspace_bytes(ta, tb, M, N, K, cus)
    if splits > 1:
        assert ws_bytes == splits * M * N * 8
    elif tail_tiles == 0:
        assert ws_bytes == 0
    A, B, C0 = pg._logical(seed, M, N, K, kind=kind)
    Ab, As = pg.stored(A, ta, pad=1)
    Bb, Bs = pg.stored(B, tb, pad=2)
    Cb, _ = pg.stored(C0, 0, pad=3)
    if beta == 0.0:
        Cb[:, :N] = np.nan   # must not be read
    dA, dB = gpu_util.to_dev(Ab), gpu_util.to_dev(Bb)
    c_ws, c_st = gpu_util.to_dev(Cb), gpu_util.to_dev(Cb)
    ws = torch.empty(max(1, ws_bytes // 8), dtype=torch.float64, device=DEV)
    binding.gemm_f64_general_ws(ta, tb, M, N, K, alpha, dA, Ab.shape[1], dB, Bb.shape[1], beta, c_ws, Cb.shape[1], ws, ws_bytes)
    torch.cuda.synchronize()
    binding.gemm_f64_general_static(ta, tb, M, N, K, alpha, dA, Ab.shape[1], dB, Bb.shape[1], beta, c_st, Cb.shape[1])
    torch.cuda.synchronize()
    return c_ws.cpu().numpy(), c_st.cpu().numpy(), ("split" if splits > 1 else "tail" if tail_tiles else "none"), (As, Bs, C0, Cb)


def test_static_scratch_matches_the_workspace_form_on_two_calls_in_a_row(gpu_device):
    # the second call is smaller than the first: it finds the first call's slabs in the scratch buffer and must
    # not be influenced by them; then larger ones again, one that is not split at all, and one whose last tiles alone
    # are computed in slices (the other use of the scratch buffer)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    calls = [((0, 0), -1.5, 0.5, (200, 200, 2049), "uniform"),
             ((0, 1), 1.0, 0.0, (64, 64, 4096), "uniform"),
             ((1, 0), 2.0, -1.0, (130, 257, 3000), "int"),
             ((1, 1), 1.0, 1.0, (33, 31, 20011), "int"),
             ((0, 0), 1.0, 1.0, (300, 520, 64), "uniform"),     # enough tiles, short k range: not split
             ((0, 0), 1.0, 1.0, (2088, 2049, 2047), "int"),     # a tail split on 256 compute units
             ((0, 1), 0.5, 2.0, (100, 70, 5001), "uniform")]
    for n, ((ta, tb), alpha, beta, (M, N, K), kind) in enumerate(calls):
        print("call %d: trans %s alpha %g beta %g shape %s %s" % (n, (ta, tb), alpha, beta, (M, N, K), kind), flush=True)
        c_ws, c_st, plan, (As, Bs, C0, Cb) = _both_ways(ta, tb, alpha, beta, M, N, K, kind, 900 + n, cus)
        expected = ["split", "split", "split", "split", "none", "tail" if cus == 256 else plan, "split"][n]
        assert plan == expected, "call %d: unexpected plan (%s)" % (n, plan)
        # same plan, same kernels: the two results are the same bits, padding of C included
        pins.assert_bitwise(c_st, c_ws, "static against workspace form, call %d" % n)
        # and both are right: against the oracle, to the bar of the general operation
        want = C0.copy()
        oracle.gemm_general_ref(ta, tb, alpha, As, Bs, beta, want)
        got = c_st[:, :N]
        if kind == "int":
            pins.assert_bitwise(np.ascontiguousarray(got), want, "static against the oracle, call %d" % n)
        else:
            gpu_util.check_tolerance(np.ascontiguousarray(got), want, oracle.general_scale(ta, tb, alpha, As, Bs, beta, C0),
                                     "static against the oracle, call %d" % n)
        from paper_2003_00532_amd import synth
        assert synth.padding_intact(c_st, N)


def test_static_scratch_limit_is_an_error_not_a_fallback(gpu_device):
    # a problem whose preferred split needs more than the fixed buffer: nothing is launched, C is untouched
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    M = N = 1536
    K = 65536
    need = binding.gemm_f64_split_k_workspace_bytes(0, 0, M, N, K, cus)
    assert need > binding.STATIC_SCRATCH_BYTES, "shape was meant to exceed the scratch buffer (needs %d)" % need
    dA = torch.zeros((M, K), dtype=torch.float64, device=DEV)
    dB = torch.zeros((K, N), dtype=torch.float64, device=DEV)
    dC = torch.full((M, N), 3.0, dtype=torch.float64, device=DEV)
    with pytest.raises(binding.GemmF64Error) as e:
        binding.gemm_f64_general_static(0, 0, M, N, K, 1.0, dA, K, dB, N, 1.0, dC, N)
    assert e.value.code == -10 and "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert bool(torch.all(dC == 3.0))
    # argument errors are reported as by the other entry points, before anything else
    with pytest.raises(binding.GemmF64Error) as e:
        binding.gemm_f64_general_static(0, 0, 4, 4, 4, 1.0, dA, 3, dB, 4, 1.0, dC, 4)
    assert e.value.code == -2
