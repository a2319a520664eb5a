"""C-ABI surface and host-side planning of top-k (no GPU, no kernel launch)."""
import ctypes
import os
import re
import subprocess

import pytest

from paper_2605_28213_amd import build as gl_build
from paper_2605_28213_amd import gemm, topk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _built():
    gl_build.build()


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "topk_lineage.h")).read()
    body = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(topk_[a-z_0-9]+)\s*\(", body))
    assert {"topk_run", "topk_query", "topk_variant_name"} <= names
    L = ctypes.CDLL(gemm.LIB_PATH)
    for n in sorted(names):
        assert hasattr(L, n), f"{n} declared in the header but not exported"
    assert topk.topk_variant_count() == topk.TOPK_VARIANT_COUNT == 3
    assert [topk.topk_variant_name(v) for v in range(3)] == ["T0_selection", "T1_radix_select", "T2_resident_coarse_refine"]
    for name, bit in topk.COND_BITS.items():
        assert topk.topk_cond_name(bit) == name
    assert topk.topk_variant_intent(1) == "radix_select" and "coarse + refine" in topk.topk_variant_intent(2)


def test_struct_layout_matches_the_header_as_plain_c(tmp_path):
    fields_d = [f[0] for f in topk.topk_desc_t._fields_]
    fields_q = [f[0] for f in topk.topk_query_t._fields_]
    prog = ['#include <stdio.h>', '#include <stddef.h>', '#include "topk_lineage.h"', 'int main(void){',
            'printf("%zu %zu\\n", sizeof(topk_desc_t), sizeof(topk_query_t));']
    prog += [f'printf("%zu\\n", offsetof(topk_desc_t, {f}));' for f in fields_d]
    prog += [f'printf("%zu\\n", offsetof(topk_query_t, {f}));' for f in fields_q]
    prog += ['return 0;}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(prog))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert [int(out[0]), int(out[1])] == [ctypes.sizeof(topk.topk_desc_t), ctypes.sizeof(topk.topk_query_t)]
    want = [getattr(topk.topk_desc_t, f).offset for f in fields_d] + [getattr(topk.topk_query_t, f).offset for f in fields_q]
    assert [int(x) for x in out[2:]] == want


def test_plans_and_refusals():
    d = topk.make_desc(64, 4096, 512)
    q0, q1, q2 = (topk.topk_query(v, d) for v in range(3))
    assert all(q.status == gemm.GEMM_OK and q.grid == 64 for q in (q0, q1, q2))
    assert (q0.threads, q0.passes) == (256, 512) and (q1.threads, q1.passes) == (256, 5) and (q2.threads, q2.passes) == (1024, 4)
    assert "11+11+10" in q2.path and "4 keys/lane" in q2.path
    assert "16 keys/lane" in topk.topk_query(2, topk.make_desc(2, 4097, 5, ld=4100)).path
    big = topk.make_desc(2, 70001, 300)
    assert topk.Query.names(topk.topk_query(0, big).violated) == ["ROW_IN_LDS"]
    assert topk.topk_query(1, big).status == gemm.GEMM_OK
    q = topk.topk_query(2, big)
    assert q.status == gemm.GEMM_ERR_PRECONDITION and "ROW_IN_REGISTERS" in topk.Query.names(q.violated)
    assert topk.Query.names(topk.topk_query(2, topk.make_desc(2, 1000, 5, ld=1001)).violated) == ["ALIGN16"]
    assert topk.Query.names(topk.topk_query(2, d, 256 + 4).violated) == ["ALIGN16"]
    assert topk.topk_run(2, d, 256 + 4, 256, 256) == gemm.GEMM_ERR_PRECONDITION


def test_argument_validation():
    def st(variant=1, **kw):
        a = dict(batch=2, n=100, k=10)
        a.update(kw)
        return topk.topk_query(variant, topk.make_desc(a["batch"], a["n"], a["k"], ld=a.get("ld", 0), flags=a.get("flags", 0))).status
    assert st() == gemm.GEMM_OK
    assert st(variant=3) == gemm.GEMM_ERR_BAD_VARIANT
    for bad in (dict(batch=-1), dict(n=-1), dict(k=-1), dict(k=101), dict(ld=99), dict(flags=1), dict(n=1 << 31, k=1)):
        assert st(**bad) == gemm.GEMM_ERR_BAD_ARG, bad
    assert st(k=0) == gemm.GEMM_OK and st(batch=0) == gemm.GEMM_OK and st(n=0, k=0) == gemm.GEMM_OK
    assert topk.topk_query(1, topk.make_desc(2, 100, 0)).grid == 0
    assert topk.topk_run(1, topk.make_desc(2, 100, 10), None, 256, 256) == gemm.GEMM_ERR_BAD_ARG
