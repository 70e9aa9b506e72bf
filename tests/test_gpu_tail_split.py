"""The tail split of gemm_*_general_ws (the last tiles of a problem computed in k slices into a workspace, then added
up) against the CPU oracle, element by element (needs an MI355X)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2003_00532_amd import binding, synth

import gpu_util
import pins
import pins_general as pg
from test_gpu_split_k import run_ws, SENTINEL

pytestmark = pytest.mark.gpu


def _plan(dtype, ta, tb, M, N, K, cus, ws_bytes=2 ** 62):
    fn = binding.gemm_f32_tail_split_plan if np.dtype(dtype) == np.float32 else binding.gemm_f64_tail_split_plan
    return fn(ta, tb, M, N, K, cus, ws_bytes)


def _check(dtype, ta, tb, alpha, beta, M, N, K, kind, seed, cus, require=True):
    isz = np.dtype(dtype).itemsize
    with pins.precision(dtype):
        variant, tiles, splits, chunk = _plan(dtype, ta, tb, M, N, K, cus)
        if require:
            assert tiles > 0 and splits > 1, "shape %s trans %s was meant to get a tail split" % ((M, N, K), (ta, tb))
        elif tiles == 0:
            return False
        names = binding.gemm_f32_variant_name if isz == 4 else binding.gemm_f64_variant_name
        bm, bn = (int(x) for x in names(variant).split("_")[1].split("x")[:2])
        elems = tiles * splits * bm * bn
        wsb = (binding.gemm_f32_split_k_workspace_bytes if isz == 4 else binding.gemm_f64_split_k_workspace_bytes)(ta, tb, M, N, K, cus)
        assert wsb == elems * isz
        A, B, C0 = pg._logical(seed, M, N, K, kind=kind)
        Ab, As = pg.stored(A, ta, pad=2)
        Bb, Bs = pg.stored(B, tb, pad=4)
        Cb, _ = pg.stored(C0, 0, pad=3)
        if beta == 0.0:
            Cb[:, :N] = np.nan       # must not be read
        c2, ws, a2, b2 = run_ws(ta, tb, alpha, Ab, Bb, beta, Cb, M, N, K, elems)
        what = "tail split of %d tiles x %d slices of %d, %s %s trans %s alpha %g beta %g" % (tiles, splits, chunk, kind, (M, N, K), (ta, tb), alpha, beta)
        print(what, flush=True)
        assert synth.padding_intact(c2, N) and synth.padding_intact(a2, As.shape[1]) and synth.padding_intact(b2, Bs.shape[1]), what
        assert np.all(ws[elems:] == SENTINEL), what + ": wrote past the workspace on offer"
        want = C0.copy()
        oracle.gemm_general_ref(ta, tb, alpha, As, Bs, beta, want)
        if kind == "int":
            pins.assert_bitwise(c2[:, :N], want, what)
        else:
            S = oracle.general_scale(ta, tb, alpha, As, Bs, beta, C0)
            gpu_util.check_tolerance(c2[:, :N], want, S, what)
    return True


@pytest.mark.parametrize("dtype", [np.float64, np.float32], ids=["f64", "f32"])
@pytest.mark.parametrize("combo", pg.COMBOS, ids=["nn", "nt", "tn", "tt"])
def test_tail_split_against_the_oracle_on_the_ragged_configuration(gpu_device, combo, dtype):
    # 2088 x 2049 x 2047: edge tiles in both directions and a ragged last K stage inside the last slice
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    ta, tb = combo
    # double precision: planned for every layout on 256 compute units; single precision: where the plan says so, and
    # 2500^3 (64 x 128 tiles) otherwise
    M, N, K = 2088, 2049, 2047
    if dtype == np.float32 and _plan(dtype, ta, tb, M, N, K, cus)[1] == 0:
        M, N, K = 2500, 2500, 2500
    for n, (kind, alpha, beta) in enumerate((("int", 1.0, 1.0), ("uniform", 1.0, 1.0), ("int", -2.0, 3.0), ("uniform", 0.75, 0.0))):
        _check(dtype, ta, tb, alpha, beta, M, N, K, kind, 700 + n, cus, require=(cus == 256))


@pytest.mark.parametrize("shape", [(2500, 2500, 2500), (4095, 4097, 4095), (2112, 2112, 2048), (4352, 4352, 1024)], ids=str)
def test_tail_split_on_other_tile_shapes(gpu_device, shape):
    # shapes whose plan uses the larger tiles (the last two have only full tiles and whole K stages: the lean kernel)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    M, N, K = shape
    if _plan(np.float64, 0, 0, M, N, K, cus)[1] == 0:
        pytest.skip("no tail split planned for %s on %d compute units" % (shape, cus))
    _check(np.float64, 0, 0, 1.0, 1.0, M, N, K, "int", 720, cus)
    _check(np.float64, 0, 0, 1.5, -0.5, M, N, K, "uniform", 721, cus)


def test_tail_split_is_repeatable_and_a_smaller_offer_is_the_plain_call(gpu_device):
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    M, N, K = 2088, 2049, 2047
    A, B, C0 = pg._logical(730, M, N, K)
    Cb, _ = pg.stored(C0, 0, pad=1)
    full = binding.gemm_f64_split_k_workspace_bytes(0, 0, M, N, K, cus) // 8
    first, _, _, _ = run_ws(0, 0, 1.0, A, B, 1.0, Cb, M, N, K, full)
    second, _, _, _ = run_ws(0, 0, 1.0, A, B, 1.0, Cb, M, N, K, full)
    pins.assert_bitwise(first, second, "two runs")
    # one element short of what the plan needs: no tail split, the workspace is not touched, the result is the
    # plain call's
    assert _plan(np.float64, 0, 0, M, N, K, cus, (full - 1) * 8)[1] == 0
    short, ws, _, _ = run_ws(0, 0, 1.0, A, B, 1.0, Cb, M, N, K, full - 1)
    assert np.all(ws == SENTINEL)
    dA, dB, dC = (gpu_util.to_dev(x) for x in (A, B, Cb))
    binding.gemm_f64_general(0, 0, M, N, K, 1.0, dA, K, dB, N, 1.0, dC, Cb.shape[1])
    torch.cuda.synchronize()
    pins.assert_bitwise(short, dC.cpu().numpy(), "short offer against the plain call")
