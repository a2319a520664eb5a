"""C-ABI surface and host-side planning of the convolution layer (no GPU, no kernel launch)."""
import ctypes
import os
import re
import subprocess

import pytest

from paper_2605_28213_amd import build as gl_build
from paper_2605_28213_amd import conv, gemm
from paper_2605_28213_amd import inputs as gen

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _built():
    gl_build.build()


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "conv_lineage.h")).read()
    body = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(conv2d_[a-z_0-9]+)\s*\(", body))
    assert {"conv2d_run", "conv2d_query", "conv2d_default_desc", "conv2d_variant_name"} <= names
    L = ctypes.CDLL(gemm.LIB_PATH)
    for n in sorted(names):
        assert hasattr(L, n), f"{n} declared in the header but not exported"
    assert conv.conv2d_variant_count() == conv.CONV_VARIANT_COUNT == 3
    assert [conv.conv2d_variant_name(v) for v in range(3)] == ["C0_direct", "C1_im2col_mfma", "C2_implicit_mfma"]
    for name, bit in conv.COND_BITS.items():
        assert conv.conv2d_cond_name(bit) == name
    assert "im2col" in conv.conv2d_variant_intent(1) and "gather" in conv.conv2d_variant_intent(2)


def test_struct_layout_matches_the_header_as_plain_c(tmp_path):
    fields_d = [f[0] for f in conv.conv2d_desc_t._fields_]
    fields_q = [f[0] for f in conv.conv2d_query_t._fields_]
    prog = ['#include <stdio.h>', '#include <stddef.h>', '#include "conv_lineage.h"', 'int main(void){',
            'printf("%zu %zu\\n", sizeof(conv2d_desc_t), sizeof(conv2d_query_t));']
    prog += [f'printf("%zu\\n", offsetof(conv2d_desc_t, {f}));' for f in fields_d]
    prog += [f'printf("%zu\\n", offsetof(conv2d_query_t, {f}));' for f in fields_q]
    prog += ['return 0;}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(prog))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert [int(out[0]), int(out[1])] == [ctypes.sizeof(conv.conv2d_desc_t), ctypes.sizeof(conv.conv2d_query_t)]
    want = [getattr(conv.conv2d_desc_t, f).offset for f in fields_d] + [getattr(conv.conv2d_query_t, f).offset for f in fields_q]
    assert [int(x) for x in out[2:]] == want


def _desc(name, **kw):
    c = gen.CONV_CONFIGS[name]
    return c, conv.make_desc(c.N, c.H, c.W, c.C, c.F, c.R, c.S, c.in_dtype, c.out_dtype, stride=c.stride, pad=c.pad, **kw)


def test_paper_layer_plans():
    c, d = _desc("CONV")
    q0, q1, q2 = (conv.conv2d_query(v, d) for v in range(3))
    for q in (q0, q1, q2):
        assert (q.P, q.Q, q.gemm_m, q.gemm_n, q.gemm_k) == (56, 56, 8 * 56 * 56, 128, 576)
    assert q0.status == gemm.GEMM_OK and q0.path == "direct" and q0.grid == 8 * 56 * 56 * 128 // 256
    # im2col: refused without scratch, and says how much it needs (the patch matrix; the filters are usable as they are)
    assert q1.status == gemm.GEMM_ERR_WORKSPACE and conv.Query.names(q1.violated) == ["SCRATCH_LENT"]
    assert q1.workspace_bytes == 8 * 56 * 56 * 576 * 2 and q1.path == "im2col+mfma32-direct-to-lds"
    assert conv.conv2d_run(1, d, 256, 256, 256) == gemm.GEMM_ERR_WORKSPACE
    d.workspace, d.workspace_bytes = 4096, q1.workspace_bytes
    assert conv.conv2d_query(1, d).status == gemm.GEMM_OK
    d.workspace_bytes -= 1
    assert conv.conv2d_query(1, d).status == gemm.GEMM_ERR_WORKSPACE
    d.workspace, d.workspace_bytes = 4100, q1.workspace_bytes          # misaligned
    assert conv.conv2d_query(1, d).status == gemm.GEMM_ERR_WORKSPACE
    # implicit: no scratch, 128 x 128 tiles over (pixels, filters), two workgroups per CU
    assert q2.status == gemm.GEMM_OK and q2.workspace_bytes == 0 and q2.violated == 0
    assert (q2.bm, q2.bn, q2.bk, q2.threads, q2.lds_bytes) == (128, 128, 64, 256, 80 * 1024)
    assert q2.grid == 8 * 56 * 56 // 128 and q2.path == "implicit-gather+mfma32-direct-to-lds"


def test_implicit_state_refuses_what_it_cannot_gather():
    c, d = _desc("CONV_c24")
    q = conv.conv2d_query(2, d)
    assert q.status == gemm.GEMM_ERR_PRECONDITION and conv.Query.names(q.violated) == ["C_WHOLE_SLABS"]
    q1 = conv.conv2d_query(1, d)                       # K = 216 is padded to 256; the filters get a padded copy
    M = c.N * c.P * c.Q
    assert q1.workspace_bytes == (M + c.F) * 256 * 2 and "pad(w)" in q1.path
    c, d = _desc("CONV")
    assert conv.Query.names(conv.conv2d_query(2, d, 256 + 8, 256, 256).violated) == ["ALIGN16_X"]
    assert conv.Query.names(conv.conv2d_query(2, d, 256, 256 + 2, 256).violated) == ["ALIGN16_W"]
    assert conv.conv2d_run(2, d, 256 + 8, 256, 256) == gemm.GEMM_ERR_PRECONDITION
    big = conv.make_desc(64, 1024, 1024, 64, 8, 3, 3, gen.F16, gen.F16, pad=(1, 1))     # 8 GiB of activations
    assert conv.Query.names(conv.conv2d_query(2, big).violated) == ["X_BELOW_2GIB"]
    f32 = conv.make_desc(1, 8, 8, 64, 8, 3, 3, gen.F32, gen.F32, pad=(1, 1))
    for v in (1, 2):
        q = conv.conv2d_query(v, f32)
        assert q.status == gemm.GEMM_ERR_PRECONDITION and "DTYPE_ON_FAST_KERNEL" in conv.Query.names(q.violated)
    assert conv.conv2d_query(0, f32).status == gemm.GEMM_OK


def test_argument_validation():
    ok = dict(N=1, H=8, W=8, C=64, F=8, R=3, S=3)
    def q(variant=0, in_dtype=gen.F16, out_dtype=gen.F16, stride=(1, 1), pad=(1, 1), flags=0, **kw):
        a = dict(ok, **kw)
        d = conv.make_desc(a["N"], a["H"], a["W"], a["C"], a["F"], a["R"], a["S"], in_dtype, out_dtype, stride=stride, pad=pad, flags=flags)
        return conv.conv2d_query(variant, d).status
    assert q() == gemm.GEMM_OK
    assert q(variant=3) == gemm.GEMM_ERR_BAD_VARIANT and q(variant=-1) == gemm.GEMM_ERR_BAD_VARIANT
    for bad in (dict(N=-1), dict(H=0), dict(C=0), dict(R=0), dict(S=300), dict(F=-2)):
        assert q(**bad) == gemm.GEMM_ERR_BAD_ARG, bad
    assert q(stride=(0, 1)) == gemm.GEMM_ERR_BAD_ARG and q(pad=(-1, 0)) == gemm.GEMM_ERR_BAD_ARG and q(flags=1) == gemm.GEMM_ERR_BAD_ARG
    assert q(H=2, pad=(0, 0)) == gemm.GEMM_ERR_BAD_ARG                  # filter larger than the image
    assert q(in_dtype=gen.F16, out_dtype=gen.BF16) == gemm.GEMM_ERR_UNSUPPORTED_DTYPE
    assert q(in_dtype=7) == gemm.GEMM_ERR_UNSUPPORTED_DTYPE
    assert q(N=0) == gemm.GEMM_OK and q(F=0) == gemm.GEMM_OK            # empty layers are legal and launch nothing
    d = conv.make_desc(1, 8, 8, 64, 8, 3, 3, gen.F16, gen.F16, pad=(1, 1))
    assert conv.conv2d_run(0, d, None, 256, 256) == gemm.GEMM_ERR_BAD_ARG
    dd = conv.conv2d_default_desc(8, 56, 56, 64, 128, 3, 3, gen.F16)
    assert (dd.pad_h, dd.pad_w, dd.stride_h, dd.stride_w, dd.out_dtype) == (1, 1, 1, 1, gen.F16)


def test_planner_properties_over_random_layers():
    """Seeded random geometries: output sizes agree with the oracle's definition, the lowered product's
    sizes are N*P*Q x F x R*S*C, the implicit state's conditions are exactly the documented ones, and
    im2col's scratch is the patch matrix (plus a padded copy of the filters when K is not whole slabs)."""
    import numpy as np
    import oracle
    rng = np.random.default_rng(0)
    es_of = {gen.F32: 4, gen.BF16: 2, gen.F16: 2, gen.E4M3: 1}
    for _ in range(300):
        dt = int(rng.choice([gen.F32, gen.BF16, gen.F16, gen.E4M3]))
        out = gen.BF16 if dt == gen.E4M3 else dt
        N, H, W = int(rng.integers(0, 5)), int(rng.integers(1, 40)), int(rng.integers(1, 40))
        C, F = int(rng.choice([3, 24, 64, 96, 128, 192])), int(rng.integers(0, 300))
        R, S = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        st, pd = (int(rng.integers(1, 4)), int(rng.integers(1, 4))), (int(rng.integers(0, 3)), int(rng.integers(0, 3)))
        d = conv.make_desc(N, H, W, C, F, R, S, dt, out, stride=st, pad=pd)
        q = [conv.conv2d_query(v, d) for v in range(3)]
        if H + 2 * pd[0] < R or W + 2 * pd[1] < S:
            assert all(x.status == gemm.GEMM_ERR_BAD_ARG for x in q)
            continue
        P, Q = oracle.conv2d_output_size(H, W, R, S, st, pd)
        es, K = es_of[dt], R * S * C
        for x in q:
            assert (x.P, x.Q, x.gemm_m, x.gemm_n, x.gemm_k) == (P, Q, N * P * Q, F, K)
        assert q[0].status == gemm.GEMM_OK and q[0].workspace_bytes == 0
        if dt == gen.F32:
            assert q[1].status == q[2].status == gemm.GEMM_ERR_PRECONDITION
            continue
        kp = -(-K * es // 128) * 128 // es
        want_ws = N * P * Q * kp * es + (F * kp * es if kp != K else 0)
        assert q[1].workspace_bytes == want_ws and q[1].status == gemm.GEMM_ERR_WORKSPACE
        ok2 = (C * es) % 128 == 0
        assert (q[2].status == gemm.GEMM_OK) == ok2
        if not ok2:
            assert conv.Query.names(q[2].violated) == ["C_WHOLE_SLABS"]
        else:
            assert q[2].workspace_bytes == 0 and (q[2].bm, q[2].bn) == (128, 128)
            assert q[2].grid == (0 if N * P * Q == 0 or F == 0 else -(-N * P * Q // 128) * -(-F // 128))
