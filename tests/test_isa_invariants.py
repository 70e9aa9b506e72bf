"""What the paper verifies by reading the generated assembly (Sections 2.8 and 2.10: no accesses to C inside the
innermost loop, no register spills, operand loads amortised over many multiply-adds), asserted on the gfx950
assembly of the double-precision kernels.  Needs hipcc, no GPU; compiles the device code once (about a minute)."""
import collections
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2003_00532_amd", "csrc", "gemm_f64.hip")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.fixture(scope="module")
def asm(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("isa") / "gemm_f64.s")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument", "--cuda-device-only", "-S", SRC, "-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    return open(out).read()


def kernels(asm_text):
    """name -> dict(vgpr, lds, scratch, body) for every gemm_mfma_kernel instantiation."""
    meta = {}
    for m in re.finditer(r"\.group_segment_fixed_size:\s*(\d+).*?\.name:\s*(\S+).*?\.private_segment_fixed_size:\s*(\d+).*?"
                         r"\.vgpr_count:\s*(\d+)", asm_text, re.S):
        lds, name, scratch, vgpr = m.groups()
        if "gemm_mfma_kernel" in name:
            meta[name] = dict(lds=int(lds), scratch=int(scratch), vgpr=int(vgpr))
    for name in meta:
        start = asm_text.index("\n" + name + ":")
        meta[name]["body"] = asm_text[start:asm_text.index(".Lfunc_end", start)]
    return meta


def params(name):
    """(BM, BN, mode, ta, tb) from the mangled name gemm_mfma_kernelIdLi<BM>ELi<BN>ELi2ELi2ELi<MODE>ELb<TA>ELb<TB>E."""
    m = re.search(r"gemm_mfma_kernelIdLi(\d+)ELi(\d+)ELi2ELi2ELi(\d)ELb(\d)ELb(\d)E", name)
    return tuple(int(x) for x in m.groups())


def mfma_blocks(body):
    blocks, cur = [], []
    for line in body.splitlines():
        t = line.strip()
        if not t or t.startswith((";", "//")):
            continue
        if re.match(r"^\.LBB\d+_\d+:", t):
            blocks.append(cur)
            cur = []
        elif not t.startswith("."):
            cur.append(t.split()[0])
    blocks.append(cur)
    return [b for b in blocks if any(op.startswith("v_mfma") for op in b)]


def test_no_kernel_spills_and_register_budgets_hold(asm):
    ks = kernels(asm)
    assert len(ks) >= 4 * 3 * 4 + 2 * 3 * 2
    for name, k in ks.items():
        bm, bn, mode, ta, tb = params(name)
        assert k["scratch"] == 0, "%s spills %d bytes" % (name, k["scratch"])
        # occupancy the selection model counts on: 128x128 two workgroups per CU, 128x64 and 64x128 three,
        # 64x64 four (512 VGPRs per SIMD lane, allocated in units of 8), thin tiles six
        budget = {128 * 128: 256, 128 * 64: 168, 64 * 64: 128, 32 * 64: 80}[bm * bn]
        assert k["vgpr"] <= budget, "%s uses %d VGPRs, more than %d" % (name, k["vgpr"], budget)
        resident = {128 * 128: 2, 128 * 64: 3, 64 * 64: 4, 32 * 64: 6}[bm * bn]
        assert resident * k["lds"] <= 160 * 1024, "%s: %d workgroups do not fit in LDS" % (name, resident)


def test_k_loop_touches_no_c_and_has_no_vector_alu_work(asm):
    for name, k in kernels(asm).items():
        bm, bn, mode, ta, tb = params(name)
        if mode != 0:
            continue  # the lean instantiation is the steady-state loop; the others add the zero-filled VGPR path
        blocks = mfma_blocks(k["body"])
        assert len(blocks) > 2, name
        ops = collections.Counter(op for b in blocks for op in b)
        assert not any(op.startswith(("global_load_dword", "global_store", "buffer_", "flat_", "scratch_")) for op in ops), \
            "%s: the MFMA blocks access memory other than through global->LDS copies: %s" % (name, dict(ops))
        # The first two blocks are the peeled first iteration of a tile (its MFMAs take a zero accumulator operand and the
        # LDS addresses are set up among them); the steady-state loop and the last iteration follow and hold next to no
        # vector-ALU instruction (the few that remain are address increments of LDS reads whose offsets exceed the
        # immediate field).
        first = collections.Counter(op for b in blocks[:2] for op in b)
        assert sum(n for op, n in first.items() if op.startswith("v_") and not op.startswith("v_mfma")) <= 24, name
        ops = collections.Counter(op for b in blocks[2:] for op in b)
        valu = sum(n for op, n in ops.items() if op.startswith("v_") and not op.startswith("v_mfma"))
        mfma = sum(n for op, n in ops.items() if op.startswith("v_mfma"))
        assert valu <= 6 and valu * 16 <= mfma, "%s: %d vector-ALU instructions among %d MFMAs" % (name, valu, mfma)
        # no register is cleared with moves: the first MFMA into every accumulator takes the constant 0 instead
        assert len(re.findall(r"v_mfma_f64_16x16x4_f64 v\[\d+:\d+\], v\[\d+:\d+\], v\[\d+:\d+\], 0\b", k["body"])) >= (bm // 32) * (bn // 32), name
        # operand fetches are amortised over the wave tile: fewer LDS reads than MFMAs even for the smallest one
        lds_reads = sum(n for op, n in ops.items() if op.startswith("ds_read"))
        assert lds_reads < mfma and ops["s_barrier"] >= 1, name


def test_every_kernel_uses_the_double_precision_matrix_instruction(asm):
    for name, k in kernels(asm).items():
        ops = collections.Counter(re.findall(r"^\s*(v_mfma\w+)", k["body"], re.M))
        assert set(ops) == {"v_mfma_f64_16x16x4_f64"}, (name, dict(ops))
