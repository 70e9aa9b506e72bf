"""Split K with a caller-provided workspace (gemm_*_general_ws) against the CPU oracle (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2003_00532_amd import binding, synth

import gpu_util
import pins
import pins_general as pg

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
DTYPES = [np.float64, np.float32]
SENTINEL = -777.25


def _ws_fn(dtype):
    return binding.gemm_f32_general_ws if np.dtype(dtype) == np.float32 else binding.gemm_f64_general_ws


def _plan_fn(dtype):
    return binding.gemm_f32_split_k_plan if np.dtype(dtype) == np.float32 else binding.gemm_f64_split_k_plan


def run_ws(ta, tb, alpha, Asb, Bsb, beta, Cb, M, N, K, ws_elems, guard=64):
    """Run with a workspace of ws_elems elements followed by a guard band; returns C and the workspace as NumPy."""
    tdt = torch.float32 if Cb.dtype == np.float32 else torch.float64
    dA, dB, dC = (gpu_util.to_dev(x) for x in (Asb, Bsb, Cb))
    ws = torch.full((ws_elems + guard,), SENTINEL, dtype=tdt, device=DEV)
    _ws_fn(Cb.dtype)(ta, tb, M, N, K, alpha, dA, Asb.shape[1], dB, Bsb.shape[1], beta, dC, Cb.shape[1], ws,
                     ws_elems * Cb.dtype.itemsize)
    torch.cuda.synchronize()
    return dC.cpu().numpy(), ws.cpu().numpy(), dA.cpu().numpy(), dB.cpu().numpy()


# few tiles, long (and ragged) k ranges, ragged M and N
SPLIT_SHAPES = [(100, 70, 5001), (64, 64, 4096), (130, 257, 3000), (33, 31, 20011), (200, 200, 2049)]


@pytest.mark.parametrize("dtype", DTYPES, ids=["f64", "f32"])
@pytest.mark.parametrize("combo", pg.COMBOS, ids=["nn", "nt", "tn", "tt"])
def test_split_k_against_the_oracle(gpu_device, combo, dtype):
    ta, tb = combo
    isz = np.dtype(dtype).itemsize
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    with pins.precision(dtype):
        for n, (M, N, K) in enumerate(SPLIT_SHAPES):
            variant, splits, chunk = _plan_fn(dtype)(ta, tb, M, N, K, cus)
            assert splits > 1, "shape %s was meant to be split" % ((M, N, K),)
            for kind, (alpha, beta) in (("int", (-3.0, 2.0)), ("int", (1.0, 0.0)), ("uniform", (0.75, -0.5)), ("uniform", (1.0, 1.0))):
                A, B, C0 = pg._logical(600 + n, M, N, K, kind=kind)
                Ab, As = pg.stored(A, ta, pad=1 + n)
                Bb, Bs = pg.stored(B, tb, pad=2)
                Cb, _ = pg.stored(C0, 0, pad=3)
                if beta == 0.0:
                    Cb[:, :N] = np.nan       # must not be read
                c2, ws, a2, b2 = run_ws(ta, tb, alpha, Ab, Bb, beta, Cb, M, N, K, splits * M * N)
                what = "split %d x %d, %s %s trans %s alpha %g beta %g" % (splits, chunk, kind, (M, N, K), combo, alpha, beta)
                assert synth.padding_intact(c2, N) and synth.padding_intact(a2, As.shape[1]) and synth.padding_intact(b2, Bs.shape[1]), what
                assert np.all(ws[splits * M * N:] == SENTINEL), what + ": wrote past the workspace on offer"
                assert not np.any(ws[:splits * M * N] == SENTINEL), what + ": a slab element was never written"
                want = C0.copy()
                oracle.gemm_general_ref(ta, tb, alpha, As, Bs, beta, want)
                if kind == "int":
                    pins.assert_bitwise(c2[:, :N], want, what)
                else:
                    S = oracle.general_scale(ta, tb, alpha, As, Bs, beta, C0)
                    gpu_util.check_tolerance(c2[:, :N], want, S, what)


def test_too_little_workspace_is_the_plain_call_bit_for_bit(gpu_device):
    M, N, K = 100, 70, 5001
    A, B, C0 = pg._logical(650, M, N, K)
    Ab, As = pg.stored(A, 0, pad=1)
    Bb, Bs = pg.stored(B, 0, pad=1)
    Cb, _ = pg.stored(C0, 0, pad=1)
    dA, dB, dC = (gpu_util.to_dev(x) for x in (Ab, Bb, Cb))
    binding.gemm_f64_general(0, 0, M, N, K, 1.5, dA, Ab.shape[1], dB, Bb.shape[1], 0.5, dC, Cb.shape[1])
    torch.cuda.synchronize()
    plain = dC.cpu().numpy()
    for ws_elems in (0, M * N, 2 * M * N - 1):
        variant, splits, _ = binding.gemm_f64_split_k_plan(0, 0, M, N, K, workspace_bytes=ws_elems * 8)
        c2, ws, _, _ = run_ws(0, 0, 1.5, Ab, Bb, 0.5, Cb, M, N, K, ws_elems)
        if splits == 1:
            pins.assert_bitwise(c2, plain, "workspace of %d elements" % ws_elems)
            assert np.all(ws == SENTINEL)
    # and with no workspace at all
    dC2 = gpu_util.to_dev(Cb)
    binding.gemm_f64_general_ws(0, 0, M, N, K, 1.5, dA, Ab.shape[1], dB, Bb.shape[1], 0.5, dC2, Cb.shape[1], None, 0)
    torch.cuda.synchronize()
    pins.assert_bitwise(dC2.cpu().numpy(), plain, "null workspace")


def test_split_k_is_repeatable_and_respects_a_smaller_offer(gpu_device):
    # the slabs are added in a fixed order: two runs agree bit for bit; a smaller offer gives fewer slices, still correct
    M, N, K = 130, 257, 3000
    A, B, C0 = pg._logical(660, M, N, K)
    Cb, _ = pg.stored(C0, 0, pad=0)
    full = binding.gemm_f64_split_k_workspace_bytes(0, 0, M, N, K, torch.cuda.get_device_properties(0).multi_processor_count) // 8
    first, _, _, _ = run_ws(0, 0, 1.0, A, B, 1.0, Cb, M, N, K, full)
    second, _, _, _ = run_ws(0, 0, 1.0, A, B, 1.0, Cb, M, N, K, full)
    pins.assert_bitwise(first, second, "two runs")
    want = C0.copy()
    oracle.gemm_general_ref(0, 0, 1.0, A, B, 1.0, want)
    S = oracle.general_scale(0, 0, 1.0, A, B, 1.0, C0)
    for ws_elems in (full, 2 * M * N, 3 * M * N):
        got, _, _, _ = run_ws(0, 0, 1.0, A, B, 1.0, Cb, M, N, K, ws_elems)
        gpu_util.check_tolerance(got, want, S, "offer of %d elements" % ws_elems)
