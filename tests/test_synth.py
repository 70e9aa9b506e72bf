"""The seeded input generators (no GEMM arithmetic, no GPU): layout independence, value ranges, and bit equality of
the torch (device-side) generator with the NumPy one."""
import numpy as np
import pytest

from paper_2003_00532_amd import synth


@pytest.mark.parametrize("dtype", [np.float64, np.float32], ids=["f64", "f32"])
def test_values_do_not_depend_on_ld_rows_generated_or_chunking(dtype):
    _, full = synth.matrix(3, synth.TAG_B, 70, 45, 45, "uniform", dtype)
    _, padded = synth.matrix(3, synth.TAG_B, 70, 45, 64, "uniform", dtype)
    assert np.array_equal(full, padded)
    part = np.empty((20, 45), dtype)
    synth.fill(part, 3, synth.TAG_B, "uniform", row0=30, chunk_rows=7)
    assert np.array_equal(part, full[30:50])
    assert full.min() >= -1.0 and full.max() < 1.0 and abs(float(full.mean())) < 0.1
    _, ints = synth.matrix(3, synth.TAG_B, 70, 45, None, "int", dtype)
    assert set(np.unique(ints)) == set(float(v) for v in range(-4, 5))
    _, other = synth.matrix(4, synth.TAG_B, 70, 45, None, "uniform", dtype)
    _, other_tag = synth.matrix(3, synth.TAG_C, 70, 45, None, "uniform", dtype)
    assert not np.array_equal(other, full) and not np.array_equal(other_tag, full)


@pytest.mark.parametrize("dtype", [np.float64, np.float32], ids=["f64", "f32"])
@pytest.mark.parametrize("kind", ["uniform", "int", "ones", "zeros"])
def test_torch_generator_gives_the_same_bits_as_the_numpy_one(dtype, kind):
    iv = np.uint32 if dtype == np.float32 else np.uint64
    for (r, c, ld, seed, tag) in [(37, 53, 60, 0, synth.TAG_A), (5, 1, 1, 7, synth.TAG_B), (300, 70, 70, 123456789, synth.TAG_C),
                                  (0, 4, 4, 1, synth.TAG_A), (3, 0, 2, 1, synth.TAG_A)]:
        want, _ = synth.matrix(seed, tag, r, c, ld, kind, dtype)
        got = synth.device_matrix(seed, tag, r, c, ld, kind, dtype, device="cpu", chunk_rows=16).numpy()
        assert got.shape == want.shape and np.array_equal(got.view(iv), want.view(iv)), (r, c, ld, seed, tag)


def test_torch_workload_inputs_match():
    w = synth.WORKLOADS["c0_256"]
    for integer in (False, True):
        host = synth.workload_inputs(w, seed=2, integer=integer)
        dev = synth.device_workload_inputs(w, seed=2, integer=integer, device="cpu")
        for h, d in zip(host, dev):
            assert np.array_equal(h.view(np.uint64), d.numpy().view(np.uint64))


def test_sample_rows_cover_tile_boundaries():
    rows = synth.sample_rows(8192, 192, seed=3)
    assert len(rows) == 192 and rows[0] == 0 and rows[-1] == 8191 and len(set(rows.tolist())) == 192
    for r in (1, 63, 64, 127, 4095, 4096, 4097, 4159, 4160, 4223, 8063, 8064, 8065, 8127, 8128, 8191):
        assert r in rows
