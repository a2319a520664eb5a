"""C-ABI surface and host-side logic (no GPU, no kernel launch)."""
import ctypes
import os
import re

import pytest

from paper_2605_28213_amd import build as gl_build
from paper_2605_28213_amd import gemm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _built():
    gl_build.build()


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "gemm_lineage.h")).read()
    body = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(gemm_[a-z_0-9]+)\s*\(", body))
    assert {"gemm_run", "gemm_run_ex", "gemm_query", "gemm_default_desc", "gemm_status_string"} <= names
    L = ctypes.CDLL(gemm.LIB_PATH)
    for n in sorted(names):
        assert hasattr(L, n), f"{n} declared in the header but not exported"
    assert gemm.gemm_variant_count() == gemm.GEMM_VARIANT_COUNT == 5
    assert gemm.gemm_abi_version() == 3


def test_struct_layout_matches_the_header_as_plain_c(tmp_path):
    """The header must compile as C, and ctypes must agree with the C compiler on every offset."""
    import subprocess
    fields_d = [f[0] for f in gemm.gemm_desc_t._fields_]
    fields_q = [f[0] for f in gemm.gemm_query_t._fields_]
    prog = ['#include <stdio.h>', '#include <stddef.h>', '#include "gemm_lineage.h"', 'int main(void){',
            'printf("%zu %zu\\n", sizeof(gemm_desc_t), sizeof(gemm_query_t));']
    prog += [f'printf("%zu\\n", offsetof(gemm_desc_t, {f}));' for f in fields_d]
    prog += [f'printf("%zu\\n", offsetof(gemm_query_t, {f}));' for f in fields_q]
    prog += ['return 0;}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(prog))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)],
                   check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert [int(out[0]), int(out[1])] == [ctypes.sizeof(gemm.gemm_desc_t), ctypes.sizeof(gemm.gemm_query_t)]
    want = [getattr(gemm.gemm_desc_t, f).offset for f in fields_d] + [getattr(gemm.gemm_query_t, f).offset for f in fields_q]
    assert [int(x) for x in out[2:]] == want


def test_names_and_strings():
    assert [gemm.gemm_variant_name(v) for v in range(5)] == [
        "K0_naive", "K1_lds_tiled", "K2_vectorized", "K3_pipelined", "K4_mfma"]
    assert gemm.gemm_status_string(gemm.GEMM_ERR_PRECONDITION).startswith("precondition")
    for name, bit in gemm.COND_BITS.items():
        assert gemm.gemm_cond_name(bit) == name
    assert "vectorize" in gemm.gemm_variant_intent(2)


def test_default_desc_layouts():
    d = gemm.gemm_default_desc(4099, 4093, 4097, gemm.GEMM_F16)
    assert (d.layout_a, d.layout_b, d.lda, d.ldb, d.ldc, d.out_dtype) == (0, 0, 4097, 4093, 4093, gemm.GEMM_F16)
    d = gemm.gemm_default_desc(8192, 8192, 8192, gemm.GEMM_BF16)
    assert (d.layout_b, d.ldb) == (gemm.GEMM_COL_MAJOR, 8192)
    d = gemm.gemm_default_desc(8, 8, 8, gemm.GEMM_FP8_E4M3)
    assert d.out_dtype == gemm.GEMM_BF16


@pytest.mark.parametrize("variant", range(5))
def test_argument_errors_return_codes_without_launching(variant):
    ok = gemm.make_desc(64, 64, 64, gemm.GEMM_BF16, gemm.GEMM_BF16, 0, 1)
    fake = 0x1000                                         # never dereferenced: every case fails validation
    cases = []
    d = gemm.make_desc(-1, 64, 64, 1, 1, 0, 1); cases.append((d, gemm.GEMM_ERR_BAD_ARG))
    d = gemm.make_desc(64, 64, 64, 1, 1, 0, 1, batch=1); d.batch = 0; cases.append((d, gemm.GEMM_ERR_BAD_ARG))
    d = gemm.make_desc(64, 64, 64, 1, 1, 0, 1, lda=63); cases.append((d, gemm.GEMM_ERR_BAD_ARG))
    d = gemm.make_desc(64, 64, 64, 1, 1, 0, 0, ldb=10); cases.append((d, gemm.GEMM_ERR_BAD_ARG))
    d = gemm.make_desc(64, 64, 64, 1, 1, 0, 1, ldc=8); cases.append((d, gemm.GEMM_ERR_BAD_ARG))
    d = gemm.make_desc(64, 64, 64, 1, 1, 2, 1); cases.append((d, gemm.GEMM_ERR_BAD_ARG))
    d = gemm.make_desc(64, 64, 64, 7, 1, 0, 1); cases.append((d, gemm.GEMM_ERR_UNSUPPORTED_DTYPE))
    d = gemm.make_desc(64, 64, 64, gemm.GEMM_F32, gemm.GEMM_BF16, 0, 0); cases.append((d, gemm.GEMM_ERR_UNSUPPORTED_DTYPE))
    d = gemm.make_desc(64, 64, 64, 1, 1, 0, 1, batch=2, stride_c=100); cases.append((d, gemm.GEMM_ERR_BAD_ARG))
    d = gemm.make_desc(64, 64, 64, 1, 1, 0, 1, flags=1 << 20); cases.append((d, gemm.GEMM_ERR_BAD_ARG))
    d = gemm.make_desc(64, 64, 64, 1, 1, 0, 1, flags=gemm.GEMM_FLAG_TILE_256 | gemm.GEMM_FLAG_TILE_128)
    cases.append((d, gemm.GEMM_ERR_BAD_ARG))
    if variant != gemm.GEMM_K4_MFMA:                       # K4-only switches on another state
        for f in (gemm.GEMM_FLAG_TILE_128, gemm.GEMM_FLAG_DEOPT_NO_SWIZZLE, gemm.GEMM_FLAG_DEOPT_NO_OVERLAP):
            cases.append((gemm.make_desc(64, 64, 64, 1, 1, 0, 1, flags=f), gemm.GEMM_ERR_BAD_ARG))
    else:                                                  # ... and on a K4 path other than the fast kernel
        cases.append((gemm.make_desc(16, 64, 64, 1, 1, 0, 1, flags=gemm.GEMM_FLAG_TILE_128), gemm.GEMM_ERR_BAD_ARG))
        cases.append((gemm.make_desc(64, 64, 60, 1, 1, 0, 1, flags=gemm.GEMM_FLAG_DEOPT_NO_SWIZZLE), gemm.GEMM_ERR_BAD_ARG))
    d = gemm.make_desc(64, 64, 64, 1, 1, 0, 1); d.reserved = 1; cases.append((d, gemm.GEMM_ERR_BAD_ARG))
    for d, want in cases:
        assert gemm.gemm_run_ex(variant, d, fake, fake, fake) == want
        assert gemm.gemm_query(variant, d).status == want
    assert gemm.gemm_run_ex(variant, ok, None, fake, fake) == gemm.GEMM_ERR_BAD_ARG
    assert gemm.gemm_run_ex(variant, ok, fake, fake, None) == gemm.GEMM_ERR_BAD_ARG
    assert gemm.lib().gemm_run_ex(variant, None, fake, fake, fake) == gemm.GEMM_ERR_BAD_ARG
    assert gemm.lib().gemm_query(variant, ctypes.byref(ok), None, None, None, None) == gemm.GEMM_ERR_BAD_ARG


def test_bad_variant():
    d = gemm.make_desc(8, 8, 8, 0, 0, 0, 0)
    for v in (-1, 5, 99):
        assert gemm.gemm_run_ex(v, d, 16, 16, 16) == gemm.GEMM_ERR_BAD_VARIANT
        assert gemm.gemm_run(v, 8, 8, 8, 0, 16, 16, 16) == gemm.GEMM_ERR_BAD_VARIANT


def test_fp32_runs_the_expert_state_on_its_masked_kernel_only():
    d = gemm.make_desc(256, 256, 256, gemm.GEMM_F32, gemm.GEMM_F32, 0, 0)
    q = gemm.gemm_query(gemm.GEMM_K4_MFMA, d)
    assert q.status == gemm.GEMM_OK and q.violated == 0 and "DTYPE_HAS_MFMA" in gemm.Query.names(q.holds)
    assert "masked" in q.path and (q.bm, q.bn, q.bk) == (64, 64, 32) and q.workspace_bytes == 0      # 4 tiles of 128: small
    strict = gemm.make_desc(256, 256, 256, gemm.GEMM_F32, gemm.GEMM_F32, 0, 0, flags=gemm.GEMM_FLAG_STRICT)
    assert gemm.gemm_query(gemm.GEMM_K4_MFMA, strict).status == gemm.GEMM_OK      # it has no faster path to insist on
    lent = gemm.make_desc(256, 256, 256, gemm.GEMM_F32, gemm.GEMM_F32, 0, 0, workspace=4096, workspace_bytes=1 << 30)
    assert "packed" not in gemm.gemm_query(gemm.GEMM_K4_MFMA, lent).path


def test_query_reports_paths_and_conditions_for_the_five_workloads():
    from paper_2605_28213_amd import inputs as gen
    def q(v, name, A=None, B=None):
        c = gen.CONFIGS[name]; lda, ldb, ldc = c.ld
        d = gemm.make_desc(c.M, c.N, c.K, c.in_dtype, c.out_dtype, c.layout_a, c.layout_b, lda=lda, ldb=ldb, ldc=ldc,
                           batch=c.batch)
        return gemm.gemm_query(v, d, A, B)
    assert q(2, "C1").path == "vec16" and q(2, "C1").violated == 0
    r = q(4, "C2"); assert r.path == "mfma32-direct-to-lds" and r.violated == 0 and (r.bm, r.bn, r.bk) == (256, 256, 64)
    assert {"TILE_DIV_M", "TILE_DIV_N", "TILE_DIV_K"} <= set(gemm.Query.names(r.holds)) and r.grid == 1024
    r = q(2, "C3"); assert r.path == "elementwise-masked" and set(gemm.Query.names(r.violated)) == {"LD16_A", "LD16_B"}
    # the ragged fp16 workload: B row-major read in place by the persistent kernel, the three rows past the last whole
    # tile by the thin kernel; nothing violated, no scratch asked for, and lent scratch changes nothing
    r = q(4, "C3"); assert r.path == "mfma32-direct-to-lds(persistent,B-row-major)+thin(M-tail)" and r.violated == 0 and r.workspace_bytes == 0
    assert "TILE_DIV_M" not in gemm.Query.names(r.holds)
    c = gen.CONFIGS["C3"]
    lent = gemm.make_desc(c.M, c.N, c.K, c.in_dtype, c.out_dtype, 0, 0, workspace=4096, workspace_bytes=1 << 30)
    assert gemm.gemm_query(4, lent).path == r.path
    # the same sizes with A column-major: no kernel reads that in place, the packed path takes it when scratch is lent
    need = gemm.gemm_query(4, gemm.make_desc(c.M, c.N, c.K, c.in_dtype, c.out_dtype, 1, 0)).workspace_bytes
    lent = gemm.make_desc(c.M, c.N, c.K, c.in_dtype, c.out_dtype, 1, 0, workspace=4096, workspace_bytes=need)
    r = gemm.gemm_query(4, lent); assert r.path == "mfma32-packed+direct-to-lds+stream(M-tail)" and "K_CONTIG_A" in gemm.Query.names(r.violated)
    # fewer than 256 tiles: the masked kernel, with the conditions it misses
    r = gemm.gemm_query(4, gemm.make_desc(1027, 1021, 1025, c.in_dtype, c.out_dtype, 0, 0))
    assert "elementwise" in r.path and "K_CONTIG_B" in gemm.Query.names(r.violated)
    r = q(4, "C4"); assert r.path.startswith("mfma16-stream") and "SMALL_M" in gemm.Query.names(r.holds)
    r = q(4, "C5"); assert r.path == "mfma32-direct-to-lds(persistent)" and r.bk == 128 and r.grid == 256    # 1024 tiles on 256 persistent workgroups
    # a misaligned base pointer breaks ALIGN16 for that operand only
    r = q(3, "C2", A=0x1002, B=0x2000)
    assert r.path == "elementwise-masked(A)+vec16(B)" and gemm.Query.names(r.violated) == ["ALIGN16_A"]
    # strict mode turns the slow path into a refusal
    c = gen.CONFIGS["C3"]
    d = gemm.make_desc(c.M, c.N, c.K, c.in_dtype, c.out_dtype, 0, 0, flags=gemm.GEMM_FLAG_STRICT)
    assert gemm.gemm_query(2, d).status == gemm.GEMM_ERR_PRECONDITION
    assert gemm.gemm_run_ex(2, d, 0x1000, 0x1000, 0x1000) == gemm.GEMM_ERR_PRECONDITION
    assert gemm.gemm_query(1, d).status == gemm.GEMM_OK          # K1 relies on nothing that C3 breaks


def test_empty_problem_is_ok_and_launches_nothing():
    d = gemm.make_desc(0, 64, 64, 1, 1, 0, 1)
    for v in range(5):
        assert gemm.gemm_run_ex(v, d, None, None, None) == gemm.GEMM_OK
        assert gemm.gemm_query(v, d).grid == 0


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(gemm, "_lib", None)
    monkeypatch.setattr(gemm, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(gemm.GemmLibraryMissing):
        gemm.gemm_variant_count()
