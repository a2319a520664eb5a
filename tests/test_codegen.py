"""Code-generation guards for the expert kernels (host only: hipcc cross-compiles without a GPU).

The hot loops of the K4 kernels rely on properties no functional test can see: accumulators that
never leave their registers, buffer resources held in scalar registers (a resource the compiler
believes to be lane-dependent is wrapped in a readfirstlane loop around every load), no scratch.
This test compiles the translation unit to assembly and checks the steady-state loop of the fast
kernel and the register budget of every K4 kernel.
"""
import os
import re
import subprocess

import pytest

from paper_2605_28213_amd import build as gl_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2605_28213_amd", "csrc", "k4_mfma.hip")


@pytest.fixture(scope="module")
def asm(tmp_path_factory):
    out = tmp_path_factory.mktemp("asm") / "k4.s"
    flags = [f for f in gl_build.FLAGS if f != "-fPIC"]
    r = subprocess.run(["hipcc", *flags, "-S", "--cuda-device-only", SRC, "-o", str(out)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    return out.read_text()


def kernel_body(asm, mangled_prefix):
    m = re.search(r"^(%s\w*):[^\n]*\n(.*?)s_endpgm" % re.escape(mangled_prefix), asm, flags=re.S | re.M)
    assert m, f"kernel {mangled_prefix} not found"
    return m.group(2)


def metadata(asm, mangled_prefix):
    for block in asm.split("  - .agpr_count:")[1:]:
        name = re.search(r"\.name:\s+(\S+)", block).group(1)
        if name.startswith(mangled_prefix):
            get = lambda k: int(re.search(r"\.%s:\s+(\d+)" % k, block).group(1))
            return {"agpr": int(block.split()[0]), "vgpr": get("vgpr_count"), "vgpr_spill": get("vgpr_spill_count"),
                    "lds": get("group_segment_fixed_size"), "scratch": get("private_segment_fixed_size")}
    raise AssertionError(mangled_prefix)


def first_inner_loop(body):
    lines = body.split("\n")
    start = next(i for i, l in enumerate(lines) if "Inner Loop Header" in l)
    end = next(i for i in range(start, len(lines)) if re.match(r"\s+s_cbranch_(vccz|vccnz|scc0|scc1)\s", lines[i]))
    return [l.split()[0] for l in lines[start:end] if l.strip() and not l.strip().startswith((";", "."))]


@pytest.mark.parametrize("dtype,mfma,per_slab", [("4BF16", "v_mfma_f32_32x32x16_bf16", 64), ("3F16", "v_mfma_f32_32x32x16_f16", 64),
                                                 ("4E4M3", "v_mfma_scale_f32_32x32x64_f8f6f4", 32)])
def test_fast_kernel_steady_state_loop(asm, dtype, mfma, per_slab):
    prefix = "_ZN2gl12k4_mfma_fastINS_7FastCfgINS_" + dtype + "ELi256ELi8ELb1ELb1ELi0ELb0ELb0E"      # the 32x32 instantiation of the expert state
    ops = first_inner_loop(kernel_body(asm, prefix))
    count = lambda name: sum(o == name for o in ops)
    # five slabs per trip round the LDS ring; 16 direct loads per slab; fragment reads are 16-byte
    assert count(mfma) == 5 * per_slab
    assert count("buffer_load_dwordx4") == 5 * 16
    assert count("ds_read_b128") == 5 * 32
    assert count("s_barrier") == 5
    # nothing but scalar bookkeeping besides: no accumulator moves, no lane-dependent resource
    # (readfirstlane loop), no scratch, no LDS writes, no plain VALU work
    for bad in ("v_accvgpr_read_b32", "v_accvgpr_write_b32", "v_readfirstlane_b32", "s_and_saveexec_b64",
                "scratch_load_dword", "scratch_store_dword", "v_mov_b32_e32", "ds_write_b128"):
        assert count(bad) == 0, bad
    meta = metadata(asm, prefix)
    assert meta["agpr"] == 256 and meta["lds"] == 160 * 1024
    assert meta["vgpr_spill"] <= 32 and meta["scratch"] <= 160      # a few values parked outside the loop at most


@pytest.mark.parametrize("dtype,mfma", [("4BF16", "v_mfma_f32_16x16x32_bf16"), ("3F16", "v_mfma_f32_16x16x32_f16")])
@pytest.mark.parametrize("pre", [0, 8])
def test_fast_kernel_steady_state_loop_with_16x16_tiles(asm, dtype, mfma, pre):
    """The two-byte types' default on 256-tiles: 8 x 8 accumulator tiles of 16 x 16 per wave, two k-steps of 64
    instructions per slab; the same loads, fragment reads and barriers as the 32x32 form."""
    prefix = "_ZN2gl12k4_mfma_fastINS_7FastCfgINS_" + dtype + "ELi256ELi8ELb1ELb1ELi%dELb0ELb1E" % pre
    ops = first_inner_loop(kernel_body(asm, prefix))
    count = lambda name: sum(o == name for o in ops)
    assert count(mfma) == 5 * 128
    assert count("buffer_load_dwordx4") == 5 * 16
    assert count("ds_read_b128") == 5 * 32
    assert count("s_barrier") == 5
    for bad in ("v_readfirstlane_b32", "s_and_saveexec_b64", "scratch_load_dword", "scratch_store_dword", "ds_write_b128"):
        assert count(bad) == 0, bad
    # (a handful of accumulator tiles change register file per slab: 256 accumulator registers and 128 of fragments)
    assert count("v_accvgpr_read_b32") + count("v_accvgpr_write_b32") <= 5 * 16
    meta = metadata(asm, prefix)
    assert meta["agpr"] == 256 and meta["lds"] == 160 * 1024 and meta["vgpr_spill"] == 0 and meta["scratch"] == 0


def test_stream_kernel_register_budget(asm):
    for dtype in ("4BF16", "3F16", "4E4M3"):
        for waves in (1, 4):
            meta = metadata(asm, "_ZN2gl9k4_streamINS_9StreamCfgINS_%sELi%dELi1ELi256ELi19ELi1EEE" % (dtype, waves))
            assert meta["vgpr_spill"] == 0 and meta["scratch"] == 0
            assert meta["lds"] == waves * 16 * 1024, "per wave the A group and one column group of 16 x 512 B"
        # 17..64 rows: (waves, column groups, K tile, groups of A); per wave MG + 1 groups of 16 x 2 TK bytes
        for waves, nb, tk, mg in ((2, 2, 256, 2), (4, 4, 128, 3), (4, 4, 128, 4), (4, 4, 128, 6)):
            meta = metadata(asm, "_ZN2gl9k4_streamINS_9StreamCfgINS_%sELi%dELi%dELi%dELi19ELi%dEEE" % (dtype, waves, nb, tk, mg))
            assert meta["vgpr_spill"] == 0 and meta["scratch"] == 0
            assert meta["lds"] == waves * (mg + 1) * 16 * 2 * tk


def test_small_tile_configuration_fits_two_workgroups_per_cu(asm):
    for dtype in ("4BF16", "3F16", "4E4M3"):
        meta = metadata(asm, "_ZN2gl12k4_mfma_fastINS_7FastCfgINS_" + dtype + "ELi128ELi8ELb1ELb1ELi0ELb0E")
        assert meta["lds"] == 80 * 1024 and meta["agpr"] + meta["vgpr"] <= 512
        assert meta["vgpr"] <= 256 and meta["vgpr_spill"] == 0, "two waves per SIMD need at most 256 registers each"


def test_gathering_instantiation_keeps_two_workgroups_per_cu(asm):
    """The convolution form of the fast kernel: same budget as the 128-tile matrix product."""
    for dtype in ("4BF16", "3F16", "4E4M3"):
        meta = metadata(asm, "_ZN2gl12k4_mfma_fastINS_7FastCfgINS_" + dtype + "ELi128ELi8ELb1ELb1ELi0ELb1E")
        assert meta["lds"] == 80 * 1024 and meta["vgpr"] <= 256 and meta["vgpr_spill"] == 0 and meta["scratch"] == 0
        body = kernel_body(asm, "_ZN2gl12k4_mfma_fastINS_7FastCfgINS_" + dtype + "ELi128ELi8ELb1ELb1ELi0ELb1E")
        assert "v_readfirstlane_b32" not in first_inner_loop(body), "the activations' buffer resource must stay scalar"


def test_static_scratch_array_is_a_visible_device_symbol(tmp_path):
    """gemm_run_static finds its scratch array through hipGetSymbolAddress, which looks the name up in the
    loaded code object: the array must be emitted as a global symbol of the declared size, 256-byte
    aligned (a symbol kept local is not found and the runtime aborts the process)."""
    src = os.path.join(ROOT, "paper_2605_28213_amd", "csrc", "gemm_api.hip")
    out = tmp_path / "api.s"
    flags = [f for f in gl_build.FLAGS if f != "-fPIC"]
    r = subprocess.run(["hipcc", *flags, "-S", "--cuda-device-only", src, "-o", str(out)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    text = out.read_text()
    header = open(os.path.join(ROOT, "include", "gemm_lineage.h")).read()
    mib = int(re.search(r"#define GEMM_STATIC_SCRATCH_BYTES \(\(size_t\)(\d+) << 20\)", header).group(1))
    m = re.search(r"\.globl\s+(\w*scratch\w*)\n\s*\.p2align\s+(\d+)", text)
    assert m, "the scratch array is not a global symbol of the device code"
    assert int(m.group(2)) >= 8
    assert re.search(r"\.size\s+%s, %d\b" % (re.escape(m.group(1)), mib << 20), text)


def test_persistent_kernel_slab_loop(tmp_path):
    """The persistent form of the 256-tile kernel: the middle-slab loop holds one slab (64 or 32 matrix instructions,
    32 fragment reads, 16 direct loads issued from inline assembly, one barrier, the one hand-placed vmcnt wait),
    nothing spills in the two-byte instantiations, and no scratch access sits between the first and the last matrix
    instruction of any instantiation (a scratch reload there would wait for the direct loads in flight)."""
    src = os.path.join(ROOT, "paper_2605_28213_amd", "csrc", "k4_ring.hip")
    out = tmp_path / "ring.s"
    flags = [f for f in gl_build.FLAGS if f != "-fPIC"] + gl_build.EXTRA_FLAGS["k4_ring.hip"]
    r = subprocess.run(["hipcc", *flags, "-S", "--cuda-device-only", src, "-o", str(out)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    text = out.read_text()
    for dtype, mfma, per_slab in (("4BF16", "v_mfma_f32_32x32x16_bf16", 64), ("3F16", "v_mfma_f32_32x32x16_f16", 64),
                                  ("4E4M3", "v_mfma_scale_f32_32x32x64_f8f6f4", 32)):
        prefix = "_ZN2gl12k4_mfma_ringINS_7RingCfgINS_" + dtype + "ELi8ELb0E"
        m = re.search(r"^(%s\w*):[^\n]*\n(.*?)\.Lfunc_end" % re.escape(prefix), text, flags=re.S | re.M)
        assert m, prefix
        ops = first_inner_loop(m.group(2))
        count = lambda name: sum(o == name for o in ops)
        assert count(mfma) == per_slab and count("ds_read_b128") == 32 and count("buffer_load_dwordx4") == 16 and count("s_barrier") == 1
        for bad in ("v_accvgpr_read_b32", "v_accvgpr_write_b32", "v_readlane_b32", "v_readfirstlane_b32", "scratch_load_dword",
                    "scratch_store_dword", "scratch_load_dwordx4", "scratch_store_dwordx4", "ds_write_b128"):
            assert count(bad) == 0, bad
        assert not any(o.startswith("v_cmp") for o in ops), "no vector instruction of the middle-slab loop writes a scalar register"
        lines = m.group(2).split("\n")
        mf = [i for i, l in enumerate(lines) if mfma in l]
        assert len(mf) == 4 * per_slab                      # the four slab kinds, each once
        assert not any(l.strip().startswith("scratch_") for l in lines[mf[0]:mf[-1]])
        meta = metadata(text, prefix)
        assert meta["agpr"] == 256 and meta["lds"] == 160 * 1024
        assert meta["vgpr_spill"] == (0 if dtype != "4E4M3" else meta["vgpr_spill"]) and meta["vgpr_spill"] <= 2
    # Every direct load issued from inline assembly keeps the wait states gfx9 does not interlock (and the compiler's
    # hazard pass does not place inside inline assembly): one after the scalar write of M0, and five after a vector
    # instruction that wrote a scalar register the load reads as descriptor or offset (a scalar spill reload is one).
    code = [l.strip() for l in text.split("\n")]
    code = [l for l in code if l and not l.startswith((";", ".", "//")) and not l.endswith(":")]
    loads = [i for i, l in enumerate(code) if l.startswith("buffer_load_dwordx4") and l.endswith("lds")]
    assert len(loads) > 100
    checked = 0
    for i in loads:
        assert code[i - 1].startswith("s_nop") and code[i - 2].startswith("s_mov_b32 m0"), code[i - 3:i + 1]
        m = re.match(r"buffer_load_dwordx4 v\d+, s\[(\d+):(\d+)\], (s\d+|vcc_lo|vcc_hi) offen lds", code[i])
        assert m, code[i]
        used = {"s%d" % r for r in range(int(m.group(1)), int(m.group(2)) + 1)} | {m.group(3)}
        waited, j = 0, i - 1
        while waited < 5 and j >= 0:
            ins = code[j]
            w = re.match(r"(v_readlane_b32|v_readfirstlane_b32) (s\d+|vcc_lo|vcc_hi),", ins)
            assert not (w and w.group(2) in used), (code[j:i + 1], "a scalar register written by a vector instruction is read %d wait states later" % waited)
            if used & {"vcc_lo", "vcc_hi"}:     # (the implicit destination of the short compare and carry forms)
                assert not re.match(r"v_(cmp|cmpx|add_co|sub_co|subrev_co|addc_co|subb_co|div_scale)", ins), code[j:i + 1]
            w = re.match(r"v_\S+ (s\[(\d+):(\d+)\]|s\d+),", ins)       # any other vector instruction with a scalar destination
            if w:
                regs = {w.group(1)} if w.group(2) is None else {"s%d" % r for r in range(int(w.group(2)), int(w.group(3)) + 1)}
                assert not (regs & used), code[j:i + 1]
            waited += (int(ins.split()[1]) + 1) if ins.startswith("s_nop") else 1
            j -= 1
        checked += 1
    assert checked == len(loads)
    # the form that reads a row-major B in place: per slab 16 fragment reads of A and 32 transposing reads of B
    for dtype, mfma in (("4BF16", "v_mfma_f32_32x32x16_bf16"), ("3F16", "v_mfma_f32_32x32x16_f16")):
        prefix = "_ZN2gl12k4_mfma_ringINS_7RingCfgINS_" + dtype + "ELi8ELb1E"
        m = re.search(r"^(%s\w*):[^\n]*\n(.*?)\.Lfunc_end" % re.escape(prefix), text, flags=re.S | re.M)
        assert m, prefix
        ops = first_inner_loop(m.group(2))
        count = lambda name: sum(o == name for o in ops)
        assert count(mfma) == 64 and count("ds_read_b128") == 16 and count("ds_read_b64_tr_b16") == 32
        assert count("buffer_load_dwordx4") == 16 and count("s_barrier") == 1
        meta = metadata(text, prefix)
        assert meta["vgpr_spill"] == 0 and meta["scratch"] == 0 and meta["lds"] == 160 * 1024
