"""Host-side logic of libgemm_f64.so that needs no GPU: exported symbols, argument validation,
variant selection and the workgroup -> tile mapping."""
import ctypes
import os
import re

import pytest

from paper_2003_00532_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = []
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if fn.endswith(".h"):
            text = open(os.path.join(inc, fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names += re.findall(r"\b(gemm_f(?:64|32)\w*)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(binding.LIB_PATH)
    names = declared_functions()
    assert "gemm_f64" in names and "gemm_f64_ex" in names and "gemm_f32" in names and len(names) >= 27
    for n in names:
        assert hasattr(lib, n), "libgemm_f64.so does not export " + n
    for n in names:
        assert hasattr(binding, n) or hasattr(binding.load(), n)


def test_version_and_variant_table():
    assert binding.gemm_f64_version() >= 100
    n = binding.gemm_f64_variant_count()
    names = [binding.gemm_f64_variant_name(v) for v in range(n)]
    assert names[0] == "naive" and len(set(names)) == n
    assert binding.gemm_f64_variant_name(n) is None and binding.gemm_f64_variant_name(-1) is None


def test_argument_validation_happens_before_any_launch():
    # every rejected call returns before the device is touched, so this runs without a GPU;
    # 0x1000 is a fake, suitably aligned, non-null address that is never dereferenced
    p = 0x1000
    raw = binding.gemm_f64_raw
    assert raw(-1, 2, 2, p, 2, p, 2, p, 2) == -1
    assert raw(2, -1, 2, p, 2, p, 2, p, 2) == -1
    assert raw(2, 2, -1, p, 2, p, 2, p, 2) == -1
    assert raw(2, 2, 3, p, 2, p, 2, p, 2) == -2
    assert raw(2, 3, 2, p, 2, p, 2, p, 3) == -3
    assert raw(2, 3, 2, p, 2, p, 3, p, 2) == -4
    assert raw(2, 2, 2, None, 2, p, 2, p, 2) == -5
    assert raw(2, 2, 2, p, 2, None, 2, p, 2) == -5
    assert raw(2, 2, 2, p, 2, p, 2, None, 2) == -5
    assert raw(2, 2, 2, p + 4, 2, p, 2, p, 2) == -6
    assert raw(2, 2, 2, p, 2, p, 2, p + 2, 2) == -6
    assert raw(2 ** 31, 2, 2, p, 2, p, 2, p, 2) == -8
    # the kernels form "tile origin + tile size" in 32-bit integers: extents within one tile of 2^31 - 1 are
    # refused (in every position, transposed or not) rather than allowed to wrap; the bound itself passes validation
    big, ok = 2 ** 31 - 128, 2 ** 31 - 129
    assert raw(big, 1, 1, p, 1, p, 1, p, 1) == -8
    assert raw(1, big, 1, p, 1, p, big, p, big) == -8
    assert raw(1, 1, big, p, big, p, 1, p, 1) == -8
    gen = binding.load().gemm_f64_general_ex
    assert gen(1, 0, big, 1, 1, 1.0, p, big, p, 1, 1.0, p, 1, None, 1) == -8
    assert gen(1, 0, ok, 1, 1, 1.0, p, ok - 1, p, 1, 1.0, p, 1, None, 1) == -2   # passes the size check, fails the next
    assert binding.load().gemm_f64_strided(big, 1, 1, 1.0, p, 1, 1, p, 1, 1, 1.0, p, 1, 1, None) == -8
    assert raw(2, 2, 2, p, 2, p, 2, p, 2, variant=99) == -9
    # empty problems succeed without touching anything, even with null pointers
    assert raw(0, 5, 5, None, 5, None, 5, None, 5) == 0
    assert raw(5, 0, 5, None, 5, None, 1, None, 1) == 0
    assert raw(5, 5, 0, None, 1, None, 5, p, 5) == 0
    for code in range(-10, 1):
        assert "unknown error" not in binding.gemm_f64_strerror(code)
    assert "unknown" in binding.gemm_f64_strerror(-1234)
    with pytest.raises(binding.GemmF64Error):
        binding.gemm_f64_ex(2, 2, 3, p, 2, p, 2, p, 2, stream=0)


@pytest.mark.parametrize("tiles", [(1, 1), (1, 9), (9, 1), (3, 5), (8, 8), (16, 16), (17, 17), (33, 7),
                                   (64, 64), (5, 100), (100, 5), (13, 29)])
def test_tile_mapping_is_a_bijection(tiles):
    tm, tn = tiles
    seen = set()
    for b in range(tm * tn):
        t = binding.gemm_f64_tile_of_block(b, tm, tn)
        assert 0 <= t[0] < tm and 0 <= t[1] < tn
        seen.add(t)
    assert len(seen) == tm * tn
    with pytest.raises(binding.GemmF64Error):
        binding.gemm_f64_tile_of_block(tm * tn, tm, tn)


def _tile_of_block_by_division(b, tiles_m, tiles_n):
    """The grouped order written with plain integer divisions (the library multiplies by host-prepared reciprocals)."""
    total = tiles_m * tiles_n
    per, rem = divmod(total, 8)
    x, s = b % 8, b // 8
    logical = x * per + min(x, rem) + s
    width = 8 * tiles_n
    g = logical // width
    first_m = g * 8
    gsz = min(tiles_m - first_m, 8)
    in_g = logical - g * width
    tn = in_g // gsz
    return first_m + in_g - tn * gsz, tn


def test_tile_mapping_equals_its_definition_by_division():
    import random
    rnd = random.Random(5)
    shapes = [(1, 1), (7, 1), (1, 7), (8, 3), (9, 3), (15, 17), (16, 16), (17, 17), (33, 33), (66, 33), (128, 256), (256, 128),
              (129, 255), (1000, 3), (3, 1000), (1, 65536), (65536, 1), (46340, 46340), (7, 306783378), (306783378, 7)]
    for tm, tn in shapes:
        total = tm * tn
        assert total < 2 ** 31
        blocks = set(range(min(total, 300))) | {total - 1 - i for i in range(min(total, 300))} | {rnd.randrange(total) for _ in range(400)}
        for b in blocks:
            assert binding.gemm_f64_tile_of_block(b, tm, tn) == _tile_of_block_by_division(b, tm, tn), (b, tm, tn)


def test_tile_mapping_keeps_an_xcd_compact():
    # 64x64 tiles (8192^2 at 128x128): the first 64 workgroups of each XCD (two per compute unit,
    # 32 compute units) must form an 8x8 patch, i.e. share 8 A panels and 8 B panels
    tm = tn = 64
    for xcd in range(8):
        tiles = [binding.gemm_f64_tile_of_block(xcd + 8 * s, tm, tn) for s in range(64)]
        rows = {t[0] for t in tiles}
        cols = {t[1] for t in tiles}
        assert len(rows) <= 8 and len(cols) <= 9


def test_variant_selection_follows_tile_quantisation():
    name = lambda M, N, K: binding.gemm_f64_variant_name(binding.gemm_f64_choose_variant(M, N, K, 256))
    # large problems: the tile with the least traffic per flop
    assert name(8192, 8192, 8192) == "mfma_128x128x16"
    # 2088 x 2049 needs 289 tiles of 128x128, two rounds on 256 compute units at ~56 % use, and 1089 of 64x64,
    # five rounds at 85 %: the 32x64 tile (2178 tiles, nine rounds at 94.5 %) wins
    assert name(2088, 2049, 2047) == "mfma_32x64x16"
    # 2048^2 as 256 tiles of 128x128 leaves every compute unit with a single workgroup
    assert name(2048, 2048, 2048) != "mfma_128x128x16"
    # a handful of tiles: what counts is the time of one tile on its own, so the smallest tile
    assert name(256, 256, 256) == "mfma_32x64x16"
    for (M, N, K) in [(1, 1, 1), (256, 256, 256), (2048, 2048, 2048), (16384, 16384, 256), (100000, 3, 7)]:
        v = binding.gemm_f64_choose_variant(M, N, K, 256)
        assert 1 <= v < binding.gemm_f64_variant_count()


def test_variant_selection_respects_the_layouts_a_variant_exists_for():
    vname = binding.gemm_f64_variant_name
    for (M, N, K) in [(256, 256, 256), (2088, 2049, 2047), (64, 64, 4096), (8192, 8192, 8192), (33, 4000, 100)]:
        for ta in (0, 1):
            for tb in (0, 1):
                for choose, nm in ((binding.gemm_f64_choose_variant_general, binding.gemm_f64_variant_name),
                                   (binding.gemm_f32_choose_variant_general, binding.gemm_f32_variant_name)):
                    v = nm(choose(ta, tb, M, N, K, 256))
                    assert not (v.startswith("mfma_32x") and ta), (v, ta, tb)
                    assert not ("x32x" in v and not tb), (v, ta, tb)
    assert vname(binding.gemm_f64_choose_variant_general(0, 0, 256, 256, 256)) == vname(binding.gemm_f64_choose_variant(256, 256, 256))
    assert binding.gemm_f64_choose_variant_general(2, 0, 256, 256, 256) == -1
    # explicit requests for a variant that does not exist for the layout are refused before any launch
    p = 0x1000
    assert binding.gemm_f64_general_raw(1, 0, 64, 64, 64, 1.0, p, 64, p, 64, 1.0, p, 64, variant=5) == -9
    assert binding.gemm_f64_general_raw(0, 0, 64, 64, 64, 1.0, p, 64, p, 64, 1.0, p, 64, variant=6) == -9


def test_single_precision_entry_points_validate_like_the_double_ones():
    p = 0x1000
    raw = binding.gemm_f32_raw
    assert raw(-1, 2, 2, p, 2, p, 2, p, 2) == -1
    assert raw(2, 2, 3, p, 2, p, 2, p, 2) == -2
    assert raw(2, 3, 2, p, 2, p, 2, p, 3) == -3
    assert raw(2, 3, 2, p, 2, p, 3, p, 2) == -4
    assert raw(2, 2, 2, None, 2, p, 2, p, 2) == -5
    assert raw(2, 2, 2, p + 2, 2, p, 2, p, 2) == -6     # 4-byte alignment is enough, 2 is not
    assert raw(2, 2, 2, p, 2, p, 2, p, 2, variant=99) == -9
    assert raw(0, 5, 5, None, 5, None, 5, None, 5) == 0
    n = binding.gemm_f32_variant_count()
    names = [binding.gemm_f32_variant_name(v) for v in range(n)]
    assert names[0] == "naive" and all(nm.endswith("x32") for nm in names[1:]) and len(names) == 7
    for (M, N, K) in [(1, 1, 1), (2048, 2048, 2048), (8192, 8192, 8192), (2088, 2049, 2047)]:
        assert 1 <= binding.gemm_f32_choose_variant(M, N, K, 256) < n


def test_general_entry_points_validate_transposed_shapes_and_folded_operands():
    p = 0x1000
    for raw, off in ((binding.gemm_f64_general_raw, 4), (binding.gemm_f32_general_raw, 2)):
        ok = lambda *a, **k: raw(*a, **k)
        # (transa, transb, M, N, K, alpha, A, lda, B, ldb, beta, C, ldc); variant 99 is rejected after
        # validation and before any launch, so a well-formed call shows up as -9 without a GPU
        assert ok(0, 0, 2, 3, 4, 1.0, p, 4, p, 3, 1.0, p, 3, variant=99) == -9
        assert ok(2, 0, 2, 3, 4, 1.0, p, 4, p, 3, 1.0, p, 3) == -1
        assert ok(0, -1, 2, 3, 4, 1.0, p, 4, p, 3, 1.0, p, 3) == -1
        assert ok(0, 0, 2, 3, 4, 1.0, p, 3, p, 3, 1.0, p, 3) == -2        # lda < K
        assert ok(1, 0, 2, 3, 4, 1.0, p, 1, p, 3, 1.0, p, 3) == -2        # transposed A is K x M: lda < M
        assert ok(1, 0, 2, 3, 4, 1.0, p, 2, p, 3, 1.0, p, 3, variant=99) == -9
        assert ok(0, 0, 2, 3, 4, 1.0, p, 4, p, 2, 1.0, p, 3) == -3        # ldb < N
        assert ok(0, 1, 2, 3, 4, 1.0, p, 4, p, 3, 1.0, p, 3) == -3        # transposed B is N x K: ldb < K
        assert ok(0, 1, 2, 3, 4, 1.0, p, 4, p, 4, 1.0, p, 3, variant=99) == -9
        assert ok(0, 0, 2, 3, 4, 1.0, p, 4, p, 3, 1.0, p, 2) == -4
        assert ok(0, 0, 2, 3, 4, 1.0, None, 4, p, 3, 1.0, p, 3) == -5
        assert ok(0, 0, 2, 3, 4, 1.0, p + off, 4, p, 3, 1.0, p, 3) == -6
        # alpha == 0 or K == 0: A and B are not read and may be null; beta == 1 then launches nothing
        assert ok(0, 0, 2, 3, 4, 0.0, None, 4, None, 3, 1.0, p, 3) == 0
        assert ok(1, 1, 2, 3, 0, 2.0, None, 2, None, 1, 1.0, p, 3) == 0
        assert ok(0, 0, 2, 3, 4, 0.0, None, 4, None, 3, 1.0, None, 3) == -5
        assert ok(0, 0, 0, 3, 4, 1.0, None, 4, None, 3, 0.0, None, 3) == 0


def test_strided_entry_points_validate_strides_before_any_launch():
    p = 0x1000
    for raw, off in ((binding.gemm_f64_strided_raw, 4), (binding.gemm_f32_strided_raw, 2)):
        # (M, N, K, alpha, A, rsa, csa, B, rsb, csb, beta, C, rsc, csc); alpha == 0 with beta == 1 passes validation
        # and launches nothing, so an accepted layout shows up as 0 without a GPU
        def call(M=2, N=3, K=4, alpha=0.0, a=p, sa=(4, 1), b=p, sb=(3, 1), beta=1.0, c=p, sc=(3, 1)):
            return raw(M, N, K, alpha, a, sa[0], sa[1], b, sb[0], sb[1], beta, c, sc[0], sc[1])
        assert call() == 0
        assert call(M=-1) == -1 and call(N=-1) == -1 and call(K=-1) == -1
        assert call(M=2 ** 31) == -8
        assert call(sa=(0, 1)) == -2 and call(sa=(4, 0)) == -2 and call(sa=(-1, 1)) == -2
        assert call(sb=(0, 1)) == -3 and call(sb=(3, -2)) == -3
        assert call(sc=(0, 1)) == -4 and call(sc=(3, 0)) == -4
        assert call(sa=(1, 1)) == 0 and call(sb=(1, 1)) == 0            # read-only operands may overlap themselves
        assert call(sc=(2, 1)) == -4 and call(sc=(1, 1)) == -4          # C may not
        assert call(sc=(1, 2)) == 0                                     # column-major C: csc >= M
        assert call(sc=(4, 2)) == -4 and call(sc=(5, 2)) == 0           # sampled rows: rsc >= csc * (N - 1) + 1
        assert call(sc=(3, 2)) == -4 and call(sc=(3, 3)) == -4 and call(sc=(3, 4)) == 0   # csc >= rsc * (M - 1) + 1
        assert call(M=1, sc=(1, 1)) == 0 and call(N=1, sc=(1, 1)) == 0  # a single row or column is always distinct
        assert call(sc=(2 ** 62, 2 ** 60)) == 0 and call(sc=(2 ** 61, 2 ** 61)) == -4     # no overflow in the check
        assert call(c=None) == -5 and call(c=p + off) == -6
        assert call(a=None, b=None) == 0                                # alpha == 0: A and B are not needed
        assert call(alpha=1.0, a=None) == -5 and call(alpha=1.0, b=None) == -5
        assert call(alpha=1.0, a=p + off) == -6 and call(alpha=1.0, b=p + off) == -6
        assert call(M=0, c=None) == 0 and call(N=0, c=None) == 0
        assert call(K=0, alpha=1.0, a=None, b=None) == 0


def test_strided_path_addresses_the_same_elements_as_the_strides():
    # the problem that the rule says will run must address, element by element, exactly what the strides address;
    # the transposed signature is claimed exactly when all three operands have a unit-stride description
    import itertools
    import numpy as np
    rng = np.random.default_rng(0)
    counts = {1: 0, 2: 0}
    sampled_c = 0

    def unit(rows, cols, rs, cs):
        return ((cs == 1 or cols == 1) and (rs >= cols or rows == 1)) or ((rs == 1 or rows == 1) and (cs >= rows or cols == 1))

    for M, N, K in itertools.product([1, 2, 3, 5], repeat=3):
        for _ in range(60):
            def pick(rows, cols):
                kind = rng.integers(6)
                if kind == 0: return (cols + int(rng.integers(3)), 1)          # row-major, maybe padded
                if kind == 1: return (1, rows + int(rng.integers(3)))          # column-major, maybe padded
                if kind == 2: return (2 * cols + 1, 2)                         # sampled rows
                if kind == 3: return (3, 3 * rows + 2)                         # sampled columns
                if kind == 4: return (1, 1)                                    # overlapping unless a vector
                return (int(rng.integers(1, 9)), int(rng.integers(1, 9)))
            (rsa, csa), (rsb, csb), (rsc, csc) = pick(M, K), pick(K, N), pick(M, N)
            try:
                path = binding.gemm_f64_strided_path(M, N, K, rsa, csa, rsb, csb, rsc, csc)
            except binding.GemmF64Error as e:
                assert e.code == -4    # only C can be rejected here: its elements would overlap
                span_r, span_c = csc * (N - 1) + 1, rsc * (M - 1) + 1
                assert M > 1 and N > 1 and rsc < span_r and csc < span_c
                continue
            i, j, k = np.arange(M)[:, None], np.arange(N)[None, :], np.arange(K)
            a_addr = i * rsa + k[None, :] * csa
            b_addr = k[:, None] * rsb + j * csb
            c_addr = i * rsc + j * csc
            assert len(set(c_addr.ravel().tolist())) == M * N, "accepted a C whose elements overlap"
            kind, swapped, ta, tb, lda, ldb, ldc, es_a, es_b, es_c = path
            counts[kind] += 1
            sampled_c += not unit(M, N, rsc, csc)
            all_unit = unit(M, K, rsa, csa) and unit(K, N, rsb, csb) and unit(M, N, rsc, csc)
            assert (kind == 1) == all_unit
            rows, cols = (N, M) if swapped else (M, N)
            x_f, x_s, kk = np.arange(rows)[:, None], np.arange(cols)[None, :], np.arange(K)
            f_addr = kk[None, :] * lda + x_f * es_a if ta else x_f * lda + kk[None, :] * es_a      # F(x, k), rows x K
            s_addr = x_s * ldb + kk[:, None] * es_b if tb else kk[:, None] * ldb + x_s * es_b      # S(k, x), K x cols
            o_addr = np.arange(rows)[:, None] * ldc + np.arange(cols)[None, :] * es_c
            if kind == 1:   # a legal call of the transposed signature
                assert (es_a, es_b, es_c) == (1, 1, 1)
                assert lda >= max(1, rows if ta else K) and ldb >= max(1, K if tb else cols) and ldc >= max(1, cols)
            if not swapped:
                assert np.array_equal(f_addr, a_addr) and np.array_equal(s_addr, b_addr) and np.array_equal(o_addr, c_addr)
            else:
                assert np.array_equal(f_addr, b_addr.T) and np.array_equal(s_addr, a_addr.T) and np.array_equal(o_addr, c_addr.T)
    assert min(counts.values()) > 200 and sampled_c > 200, (counts, sampled_c)
    # the conventional cases by name
    path = binding.gemm_f64_strided_path
    assert path(100, 80, 60, 60, 1, 80, 1, 80, 1) == (1, False, 0, 0, 60, 80, 80, 1, 1, 1)          # all row-major
    assert path(100, 80, 60, 1, 100, 1, 60, 1, 100) == (1, True, 0, 0, 60, 100, 100, 1, 1, 1)       # all column-major
    assert path(100, 80, 60, 1, 100, 80, 1, 80, 1) == (1, False, 1, 0, 100, 80, 80, 1, 1, 1)        # A^T B
    assert path(100, 80, 60, 128, 2, 80, 1, 80, 1) == (2, False, 0, 0, 128, 80, 80, 2, 1, 1)        # sampled A
    assert path(100, 80, 60, 60, 1, 80, 1, 2 * 80, 2) == (2, False, 0, 0, 60, 80, 160, 1, 1, 2)     # sampled C
    assert path(100, 80, 60, 60, 1, 80, 1, 2, 2 * 100) == (2, True, 1, 1, 80, 60, 200, 1, 1, 2)     # sampled column-major C


def test_device_peak_query_fails_cleanly_without_a_device():
    import ctypes as ct
    cus, khz, p64, p32 = ct.c_int(-5), ct.c_int(-5), ct.c_double(-5), ct.c_double(-5)
    rc = binding.load().gemm_f64_device_peak(ct.byref(cus), ct.byref(khz), ct.byref(p64), ct.byref(p32))
    assert rc in (0, -7)
    if rc == 0:
        assert cus.value > 0 and khz.value > 0 and abs(p32.value - 2 * p64.value) < 1e-9
        assert abs(p64.value - cus.value * 4 * 32 * khz.value * 1e3 / 1e12) < 1e-9
    else:
        assert (cus.value, khz.value, p64.value, p32.value) == (-5, -5, -5.0, -5.0)   # outputs untouched on failure
    assert binding.load().gemm_f64_device_peak(None, None, None, None) == rc


def test_split_k_plan_is_a_consistent_pure_function():
    for plan, stage, nm in ((binding.gemm_f64_split_k_plan, 16, binding.gemm_f64_variant_name),
                            (binding.gemm_f32_split_k_plan, 32, binding.gemm_f32_variant_name)):
        for (M, N, K) in [(640, 640, 8192), (512, 512, 4096), (128, 128, 65536), (64, 64, 1000003), (100, 70, 5001),
                          (256, 256, 256), (2048, 2048, 2048), (8192, 8192, 8192), (2088, 2049, 2047), (1, 1, 1), (0, 5, 7)]:
            for ta in (0, 1):
                for tb in (0, 1):
                    v, splits, chunk = plan(ta, tb, M, N, K)
                    assert plan(ta, tb, M, N, K) == (v, splits, chunk)
                    assert splits >= 1 and nm(v) is not None and nm(v) != "naive"
                    assert not (nm(v).startswith("mfma_32x") and ta) and not ("x32x" in nm(v) and not tb)
                    if splits == 1:
                        assert chunk == K
                    else:
                        assert chunk % stage == 0 and (splits - 1) * chunk < K <= splits * chunk
    # few tiles and a long k range are split; the benchmark configurations are not
    assert binding.gemm_f64_split_k_plan(0, 0, 640, 640, 8192)[1] > 1
    assert binding.gemm_f64_split_k_plan(0, 0, 128, 128, 65536)[1] > 1
    for (M, N, K) in [(256, 256, 256), (2048, 2048, 2048), (2088, 2049, 2047), (8192, 8192, 8192), (16384, 16384, 256)]:
        assert binding.gemm_f64_split_k_plan(0, 0, M, N, K)[1] == 1
        if (M, N, K) != (2088, 2049, 2047):   # the ragged configuration gets a tail split instead, see below
            assert binding.gemm_f64_split_k_workspace_bytes(0, 0, M, N, K) == 0
    # the workspace on offer bounds the number of slabs; none at all means no split
    M, N, K = 640, 640, 8192
    want = binding.gemm_f64_split_k_workspace_bytes(0, 0, M, N, K)
    v, splits, chunk = binding.gemm_f64_split_k_plan(0, 0, M, N, K)
    assert want == splits * M * N * 8
    for ws in (0, M * N * 8, 2 * M * N * 8, 3 * M * N * 8 + 7, want - 1, want):
        s2 = binding.gemm_f64_split_k_plan(0, 0, M, N, K, workspace_bytes=ws)[1]
        assert s2 * M * N * 8 <= ws or s2 == 1
    assert binding.gemm_f64_split_k_plan(0, 0, M, N, K, workspace_bytes=0)[1] == 1
    assert binding.load().gemm_f64_split_k_plan(2, 0, 8, 8, 8, 256, 0, None, None, None) == -1
    assert binding.load().gemm_f64_split_k_plan(0, 0, -1, 8, 8, 256, 0, None, None, None) == -1


def test_tail_split_plan_is_a_consistent_pure_function():
    for plan, ws_bytes, split_plan, nm, isz in (
            (binding.gemm_f64_tail_split_plan, binding.gemm_f64_split_k_workspace_bytes, binding.gemm_f64_split_k_plan, binding.gemm_f64_variant_name, 8),
            (binding.gemm_f32_tail_split_plan, binding.gemm_f32_split_k_workspace_bytes, binding.gemm_f32_split_k_plan, binding.gemm_f32_variant_name, 4)):
        stage = 128 // isz
        for (M, N, K) in [(2088, 2049, 2047), (2500, 2500, 2500), (4095, 4097, 4095), (2112, 2112, 2048), (4352, 4352, 1024),
                          (2048, 2048, 2048), (8192, 8192, 8192), (16384, 16384, 256), (256, 256, 256), (640, 640, 8192), (3000, 3000, 40),
                          (1, 1, 1), (0, 5, 7)]:
            for ta in (0, 1):
                for tb in (0, 1):
                    for cus in (256, 304, 64):
                        v, tiles, s, chunk = plan(ta, tb, M, N, K, cus)
                        assert plan(ta, tb, M, N, K, cus) == (v, tiles, s, chunk)
                        if tiles == 0:
                            assert s == 1 and chunk == 0
                            if split_plan(ta, tb, M, N, K, cus)[1] == 1:
                                assert ws_bytes(ta, tb, M, N, K, cus) == 0
                            continue
                        assert split_plan(ta, tb, M, N, K, cus)[1] == 1, "the two splits are never combined"
                        bm, bn = (int(x) for x in nm(v).split("_")[1].split("x")[:2])
                        total = -(-M // bm) * -(-N // bn)
                        assert 0 < tiles < total and 2 <= s <= 32
                        assert chunk % stage == 0 and (s - 1) * chunk < K <= s * chunk, "every slice has work"
                        assert ws_bytes(ta, tb, M, N, K, cus) == tiles * s * bm * bn * isz
                        # the units fit the slots of one round, which is the point of the split
                        assert tiles * s <= cus * 6
                        # one byte less than needed: a different plan (or none), never an overrun
                        v2, t2, s2, c2 = plan(ta, tb, M, N, K, cus, tiles * s * bm * bn * isz - 1)
                        if t2:
                            bm2, bn2 = (int(x) for x in nm(v2).split("_")[1].split("x")[:2])
                            assert t2 * s2 * bm2 * bn2 * isz <= tiles * s * bm * bn * isz - 1
    # the ragged benchmark configuration is the case it was built for; the others fill whole rounds or are too small
    assert binding.gemm_f64_tail_split_plan(0, 0, 2088, 2049, 2047)[1:3] == (65, 15)
    for (M, N, K) in [(256, 256, 256), (2048, 2048, 2048), (8192, 8192, 8192), (16384, 16384, 256)]:
        assert binding.gemm_f64_tail_split_plan(0, 0, M, N, K)[1] == 0
    assert binding.load().gemm_f64_tail_split_plan(2, 0, 8, 8, 8, 256, 0, None, None, None, None) == -1


def test_workspace_arguments_are_validated_before_any_launch():
    p = 0x1000
    raw = binding.load().gemm_f64_general_ws
    # an empty output (M = 0) passes the operand checks with null operands, which isolates the workspace checks
    empty = lambda ws, nbytes: raw(0, 0, 0, 3, 4, 1.0, None, 4, None, 3, 1.0, None, 3, ws, nbytes, None)
    assert empty(None, 0) == 0
    assert empty(None, 64) == -5          # bytes on offer but no pointer
    assert empty(p + 4, 64) == -6         # not aligned to the element
    assert empty(p, -1) == -5
    assert empty(p, 64) == 0


def test_gflops_convention_matches_the_papers_printed_numbers():
    # GFLOPS = 2 M N K / t / 1e9 reproduces the figures printed next to the run times (Section 1.3)
    path = os.path.join(ROOT, "tests", "golden", "paper_gflops_convention.txt")
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            name, M, N, K, secs, gflops = line.split()
            got = 2.0 * int(M) * int(N) * int(K) / float(secs) / 1e9
            assert abs(got - float(gflops)) < 0.006, (name, got)
    w = synth.WORKLOADS["c3_8192"]
    assert w.flops == 2.0 * 8192 ** 3 and w.algorithmic_bytes == 8.0 * 4 * 8192 ** 2
