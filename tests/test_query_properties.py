"""Property tests of the host-side planner (gemm_query never launches, so no GPU is needed).

For arbitrary valid descriptors: the condition masks are consistent, STRICT turns exactly the calls
with violated conditions into refusals, the reported scratch follows the packed layout, tile and
simplification switches are accepted only where they mean something, and the launch geometry covers
the problem.
"""
import math

from hypothesis import given, settings, strategies as st

from paper_2605_28213_amd import gemm

DT = st.sampled_from([gemm.GEMM_F32, gemm.GEMM_BF16, gemm.GEMM_F16, gemm.GEMM_FP8_E4M3])
LAYOUT = st.sampled_from([gemm.GEMM_ROW_MAJOR, gemm.GEMM_COL_MAJOR])
ES = {gemm.GEMM_F32: 4, gemm.GEMM_BF16: 2, gemm.GEMM_F16: 2, gemm.GEMM_FP8_E4M3: 1}


@st.composite
def descriptors(draw):
    M, N, K = draw(st.integers(1, 5000)), draw(st.integers(1, 5000)), draw(st.integers(1, 5000))
    dt = draw(DT)
    la, lb = draw(LAYOUT), draw(LAYOUT)
    out = gemm.GEMM_BF16 if dt == gemm.GEMM_FP8_E4M3 else dt
    pad = draw(st.sampled_from([0, 0, 1, 3, 8, 16]))
    lda = (K if la == gemm.GEMM_ROW_MAJOR else M) + pad
    ldb = (N if lb == gemm.GEMM_ROW_MAJOR else K) + pad
    return dict(M=M, N=N, K=K, dt=dt, out=out, la=la, lb=lb, lda=lda, ldb=ldb, ldc=N + pad, batch=draw(st.integers(1, 4)))


def make(p, **kw):
    return gemm.make_desc(p["M"], p["N"], p["K"], p["dt"], p["out"], p["la"], p["lb"], lda=p["lda"], ldb=p["ldb"],
                          ldc=p["ldc"], batch=p["batch"], **kw)


@settings(max_examples=300, deadline=None)
@given(descriptors(), st.integers(0, 4))
def test_masks_status_and_geometry_are_consistent(p, variant):
    q = gemm.gemm_query(variant, make(p))
    assert q.status in (gemm.GEMM_OK, gemm.GEMM_ERR_PRECONDITION)
    assert q.violated == q.required & ~q.holds
    assert q.status == gemm.GEMM_OK                                     # every violation has a slow path of the same state
    strict = gemm.gemm_query(variant, make(p, flags=gemm.GEMM_FLAG_STRICT))
    assert (strict.status == gemm.GEMM_ERR_PRECONDITION) == (q.violated != 0)
    assert strict.path == q.path and strict.violated == q.violated
    if q.status == gemm.GEMM_OK:
        assert q.path and q.threads in (64, 128, 256, 512) and q.grid >= 1
        if q.bm and q.bn and "stream" not in q.path and "thin" not in q.path:
            assert q.grid >= math.ceil(p["M"] / q.bm) * math.ceil(p["N"] / q.bn) * p["batch"] or "M-tail" in q.path or \
                    ("persistent" in q.path and q.grid == 256)      # (256 workgroups walking several tiles each)
        assert q.lds_bytes <= 160 * 1024


@settings(max_examples=300, deadline=None)
@given(descriptors())
def test_expert_state_paths_and_scratch(p):
    es = ES[p["dt"]]
    q = gemm.gemm_query(gemm.GEMM_K4_MFMA, make(p))
    if p["dt"] == gemm.GEMM_F32:
        # fp32 runs its matrix instruction in the masked kernel only: no fast, packed or streaming form, no scratch
        assert q.status == gemm.GEMM_OK and "masked" in q.path and q.workspace_bytes == 0 and q.violated == 0
        assert (q.bm, q.bn) in ((128, 128), (64, 64)) and q.bk == 32
        return
    fast_ok = (p["la"] == gemm.GEMM_ROW_MAJOR and p["lb"] == gemm.GEMM_COL_MAJOR and (p["lda"] * es) % 16 == 0
               and (p["ldb"] * es) % 16 == 0 and (p["batch"] == 1 or ((p["M"] * p["lda"] * es) % 16 == 0 and (p["N"] * p["ldb"] * es) % 16 == 0)))
    kvec, kslab = 16 // es, 128 // es
    cols = 16 if p["M"] <= 16 else 32 if p["M"] <= 32 else 64
    streams = p["M"] <= 16 or (p["M"] <= 96 and math.ceil(p["N"] / cols) * p["batch"] >= 128)
    group_rows = lambda r: 16 if r <= 16 else 32 if r <= 32 else 48 if r <= 48 else 64 if r <= 64 else 96   # rows a form holds
    if fast_ok and streams and p["K"] % kvec == 0:
        assert q.path == "mfma16-stream(small-M)" and q.workspace_bytes == 0
        assert q.bn == cols and q.bm == group_rows(p["M"]) and q.grid == math.ceil(p["N"] / cols) * p["batch"]
    elif (fast_ok and p["K"] % kvec == 0 and p["M"] > p["N"] and p["N"] <= 96
          and (p["N"] <= 16 or math.ceil(p["M"] / (32 if p["N"] <= 32 else 64)) * p["batch"] >= 128)):
        # few columns: the streaming kernel on the transposed product, strips along M
        strip = 16 if p["N"] <= 16 else 32 if p["N"] <= 32 else 64
        assert q.path == "mfma16-stream(small-N)" and q.workspace_bytes == 0
        assert q.bm == strip and q.bn == group_rows(p["N"]) and q.grid == math.ceil(p["M"] / strip) * p["batch"]
    elif fast_ok and p["K"] % kslab == 0:
        assert q.path.startswith("mfma32-direct-to-lds") and q.violated == 0
        # split-K: offered (through workspace_bytes) when the product has few tiles and a long K, taken when scratch is lent
        nslab, tiles = p["K"] // kslab, math.ceil(p["M"] / 128) * math.ceil(p["N"] / 128)
        # a thin row remainder goes to the streaming kernel when that saves a round of 256 tiles of 256 x 256
        t256 = math.ceil(p["M"] / 256) * math.ceil(p["N"] / 256) * p["batch"]
        t128 = math.ceil(p["M"] / 128) * math.ceil(p["N"] / 128) * p["batch"]
        small = math.ceil(t128 / 512) * (8 if es == 1 else 7) < math.ceil(t256 / 256) * 10
        per_row, rows = math.ceil(p["N"] / 256) * p["batch"], p["M"] // 256
        tail = (p["M"] > 256 and 1 <= p["M"] % 256 <= 64 and p["N"] <= 16384 and not small
                and math.ceil(rows * per_row / 256) < math.ceil((rows + 1) * per_row / 256))
        assert ("M-tail" in q.path) == tail
        splits = 1
        if p["batch"] == 1 and p["M"] > 16 and not tail and tiles < 256:
            for s_ in range(2, 9):
                if nslab % s_ == 0 and nslab // s_ >= 16 and tiles * s_ <= 640:
                    splits = s_
        assert q.workspace_bytes == (splits * p["M"] * p["N"] * 4 if splits > 1 else 0)
        assert "splitK" not in q.path
        if splits > 1:
            lent = gemm.gemm_query(gemm.GEMM_K4_MFMA, make(p, workspace=4096, workspace_bytes=q.workspace_bytes))
            assert lent.status == gemm.GEMM_OK and lent.path == "mfma32-direct-to-lds+splitK(%d)" % splits
            assert lent.grid == q.grid * splits
            small = gemm.gemm_query(gemm.GEMM_K4_MFMA, make(p, workspace=4096, workspace_bytes=q.workspace_bytes - 1))
            assert small.status == gemm.GEMM_ERR_WORKSPACE
    elif (p["dt"] in (gemm.GEMM_BF16, gemm.GEMM_F16) and p["la"] == gemm.GEMM_ROW_MAJOR and p["lb"] == gemm.GEMM_ROW_MAJOR
          and math.ceil(p["M"] / 256) * math.ceil(p["N"] / 256) * p["batch"] >= 256 and math.ceil(p["K"] / kslab) >= 3
          and p["lda"] * es <= 1 << 22 and p["K"] * p["ldb"] * es < 1 << 31):
        # both operands row-major and at least 256 tiles: the persistent kernel reads them in place, whatever their
        # alignment and K; nothing violated, no scratch asked for or used
        # a thin remainder of rows that would cost a round of tiles goes to the thin kernel (which also reads B in place)
        per_row, rows = math.ceil(p["N"] / 256) * p["batch"], p["M"] // 256
        thin_tail = (p["M"] > 256 and 1 <= p["M"] % 256 <= 64 and p["N"] <= 16384 and rows * per_row >= 256
                     and (p["K"] + 64) * p["ldb"] * 2 < 1 << 31
                     and math.ceil(rows * per_row / 256) < math.ceil((rows + 1) * per_row / 256))
        assert q.path == "mfma32-direct-to-lds(persistent,B-row-major)" + ("+thin(M-tail)" if thin_tail else "")
        assert q.violated == 0 and q.grid == 256
        assert q.workspace_bytes == 0
        lent = gemm.gemm_query(gemm.GEMM_K4_MFMA, make(p, workspace=4096, workspace_bytes=1 << 30))
        assert lent.status == gemm.GEMM_OK and lent.path == q.path
    elif (p["dt"] in (gemm.GEMM_BF16, gemm.GEMM_F16) and p["la"] == gemm.GEMM_ROW_MAJOR and p["lb"] == gemm.GEMM_ROW_MAJOR
          and p["M"] <= 64 and (p["K"] + 64) * p["ldb"] * 2 < 1 << 31 and p["M"] * p["lda"] * 2 < 1 << 31):
        # at most 64 rows, both operands row-major: the thin kernel reads B once, in place; no scratch, lent or not
        assert q.path == "mfma16-thin(B-row-major)" and q.violated == 0 and q.workspace_bytes == 0
        cols = 64
        assert q.grid == math.ceil(p["N"] / cols) * p["batch"] and q.bn == cols and q.bm >= min(p["M"], 64) and q.threads == 512
        lent = gemm.gemm_query(gemm.GEMM_K4_MFMA, make(p, workspace=4096, workspace_bytes=1 << 30))
        assert lent.path == q.path
    else:
        kp = math.ceil(p["K"] / kslab) * kslab
        assert q.path.startswith("mfma32-") and "packed" not in q.path
        # an operand that meets the fast kernel's conditions by itself is used in place, the other one is packed
        whole = p["K"] % kslab == 0
        a_ok = (whole and p["la"] == gemm.GEMM_ROW_MAJOR and (p["lda"] * es) % 16 == 0 and p["lda"] * es <= 1 << 22
                and (p["batch"] == 1 or (p["M"] * p["lda"] * es) % 16 == 0))
        b_ok = (whole and p["lb"] == gemm.GEMM_COL_MAJOR and (p["ldb"] * es) % 16 == 0 and p["ldb"] * es <= 1 << 22
                and (p["batch"] == 1 or (p["N"] * p["ldb"] * es) % 16 == 0))
        assert not (a_ok and b_ok)
        assert q.workspace_bytes == p["batch"] * ((0 if a_ok else p["M"]) + (0 if b_ok else p["N"])) * kp * es
        lent = gemm.gemm_query(gemm.GEMM_K4_MFMA, make(p, workspace=4096, workspace_bytes=q.workspace_bytes))
        tag = "(B)" if a_ok else "(A)" if b_ok else ""
        assert lent.status == gemm.GEMM_OK and lent.path.startswith("mfma32-packed%s+direct-to-lds" % tag)
        small = gemm.gemm_query(gemm.GEMM_K4_MFMA, make(p, workspace=4096, workspace_bytes=q.workspace_bytes - 1))
        assert small.status == gemm.GEMM_ERR_WORKSPACE
        odd = gemm.gemm_query(gemm.GEMM_K4_MFMA, make(p, workspace=4100, workspace_bytes=q.workspace_bytes))
        assert odd.status == gemm.GEMM_ERR_WORKSPACE


@settings(max_examples=200, deadline=None)
@given(descriptors(), st.integers(0, 4), st.sampled_from([gemm.GEMM_FLAG_TILE_128, gemm.GEMM_FLAG_TILE_256,
                                                         gemm.GEMM_FLAG_DEOPT_NO_SWIZZLE, gemm.GEMM_FLAG_DEOPT_NO_OVERLAP,
                                                         gemm.GEMM_FLAG_DEOPT_NO_RASTER, gemm.GEMM_FLAG_MFMA_32X32]))
def test_expert_only_switches_are_refused_elsewhere(p, variant, flag):
    plain = gemm.gemm_query(variant, make(p))
    q = gemm.gemm_query(variant, make(p, flags=flag))
    on_fast_kernel = (variant == gemm.GEMM_K4_MFMA and plain.status == gemm.GEMM_OK and plain.path.startswith("mfma32-direct-to-lds")
                      and "B-row-major" not in plain.path)      # (the in-place form has no simplified states: with a switch the masked kernel keeps the product)
    if on_fast_kernel:
        assert q.status == gemm.GEMM_OK
        if flag == gemm.GEMM_FLAG_TILE_128:
            assert (q.bm, q.bn) == (128, 128)
        if flag in (gemm.GEMM_FLAG_TILE_256, gemm.GEMM_FLAG_DEOPT_NO_SWIZZLE, gemm.GEMM_FLAG_DEOPT_NO_OVERLAP):
            assert (q.bm, q.bn) == (256, 256)
        if flag == gemm.GEMM_FLAG_DEOPT_NO_RASTER:
            assert (q.bm, q.bn) == (plain.bm, plain.bn) and q.path.endswith("-noraster")     # the tile walk is independent of the tile
    elif plain.status == gemm.GEMM_OK:
        assert q.status == gemm.GEMM_ERR_BAD_ARG


@settings(max_examples=150, deadline=None)
@given(descriptors(), st.integers(0, 4))
def test_vector_load_simplification_belongs_to_k2_and_k3(p, variant):
    q = gemm.gemm_query(variant, make(p, flags=gemm.GEMM_FLAG_DEOPT_NO_VECTOR))
    if variant in (gemm.GEMM_K2_VECTORIZED, gemm.GEMM_K3_PIPELINED):
        assert q.status == gemm.GEMM_OK and q.path == "elementwise-masked(-novec)"
        both = gemm.gemm_query(variant, make(p, flags=gemm.GEMM_FLAG_DEOPT_NO_VECTOR | gemm.GEMM_FLAG_DEOPT_NO_RASTER))
        assert both.status == gemm.GEMM_ERR_BAD_ARG
    else:
        assert q.status == gemm.GEMM_ERR_BAD_ARG
