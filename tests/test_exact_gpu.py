"""Bit-exact parity of every code path of the expert state (K4) with the CPU oracle, through the C ABI.

Operand entries are integers in {-2..2} (exact in bf16, fp16 and e4m3) and the output is fp32: every
partial sum of every summation order is an integer below 2^24, so a correct fp32-accumulating kernel
must reproduce the oracle's product bit for bit.  A dropped, doubled or misplaced K slab, a wrong
fragment, a stale LDS region or a mis-stored element cannot hide under a tolerance here.

Each case names the code path it is meant for and asserts, through gemm_query, that the planner takes
it: the direct-to-LDS kernel with 256- and 128-tiles (K long enough that the steady-state ring loop
runs several trips and leaves through the tail loop), its split-K form, the packed path in every
layout pair, the row-remainder split, every form of the streaming kernel (16 rows, 16 rows with K
split over waves, 32, 48, 64, 96 rows, few columns), the simplified expert states, and the headline
workload's shape at full size.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_28213_amd import gemm
from paper_2605_28213_amd import inputs as gen
from tests import util

pytestmark = pytest.mark.gpu

ROW, COL = gen.ROW_MAJOR, gen.COL_MAJOR
K4 = gemm.GEMM_K4_MFMA
DTYPES = [gen.BF16, gen.F16, gen.E4M3]


def int_inputs(dtype, M, N, K, la=ROW, lb=COL, *, batch=1, lda=0, ldb=0, ldc=0, seed=0, biased=False):
    """Operands with integer entries in {-2..2}, laid out as the descriptor says; gaps between rows
    (leading dimension beyond the extent) hold 3, which a kernel reading them would add in."""
    cfg = gen.Config("ints", M, N, K, dtype, gen.F32, la, lb, "uniform", batch=batch, lda=lda, ldb=ldb, ldc=ldc, biased=biased)
    lda, ldb, ldc = cfg.ld
    rows_a, ext_a = (M, K) if la == ROW else (K, M)
    rows_b, ext_b = (K, N) if lb == ROW else (N, K)
    rng = np.random.default_rng(1000 + seed)

    def draw(rows, ext, ld):
        x = np.full((batch, rows, ld), 3.0, dtype=np.float32)
        x[:, :, :ext] = rng.integers(-2, 3, (batch, rows, ext)).astype(np.float32)
        return gen.quantise(dtype, x.reshape(-1))
    A, B = draw(rows_a, ext_a, lda), draw(rows_b, ext_b, ldb)
    bias = rng.integers(-5, 6, N).astype(np.float32) if biased else None
    return gen.Inputs(cfg, seed, A, B, lda, ldb, ldc, rows_a * lda, rows_b * ldb, M * ldc, None, None, bias)


def oracle_for(inp):
    c = inp.cfg
    return oracle.gemm(c.in_dtype, c.layout_a, c.layout_b, c.M, c.N, c.K, inp.A, inp.lda, inp.B, inp.ldb, batch=c.batch,
                       stride_a=inp.stride_a, stride_b=inp.stride_b, bias=inp.bias)


def run_exact(inp, path, *, flags=0, lend=False, exact_path=True):
    """Runs K4 on `inp`, asserts the planner's path, and compares every output with the oracle bit for bit."""
    c = inp.cfg
    d = gemm.make_desc(c.M, c.N, c.K, c.in_dtype, gen.F32, c.layout_a, c.layout_b, lda=inp.lda, ldb=inp.ldb, ldc=inp.ldc,
                       batch=c.batch, stride_a=inp.stride_a, stride_b=inp.stride_b, stride_c=inp.stride_c, flags=flags)
    q = gemm.gemm_query(K4, d)
    if lend:
        assert q.workspace_bytes > 0, (q.path, "asks for no scratch")
        d.workspace, d.workspace_bytes = 4096, q.workspace_bytes        # any aligned non-null address: query only
        q = gemm.gemm_query(K4, d)
    assert (q.path == path) if exact_path else (path in q.path), (q.path, path, (c.M, c.N, c.K, c.batch))
    C_ref, _ = oracle_for(inp)
    rc, C, _ = util.run_config(K4, inp, flags=flags, lend_workspace=lend)
    assert rc == gemm.GEMM_OK, gemm.gemm_status_string(rc)
    np.testing.assert_array_equal(C[:, :, : c.N], C_ref, err_msg=f"{q.path} {(c.M, c.N, c.K, c.batch)}")
    return q


def slabs(dtype, n):
    """K of n whole 128-byte slabs."""
    return n * 128 // gen.ELEM_BYTES[dtype]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("tile_flag,bm", [(gemm.GEMM_FLAG_TILE_256, 256), (gemm.GEMM_FLAG_TILE_128, 128), (0, 0)])
def test_direct_to_lds_kernel_is_exact(dtype, tile_flag, bm):
    """M and N cross tile edges and end inside a tile; 24 slabs: first slab, four trips of the five-slab
    ring loop, three slabs of tail.  Also 7 and 11 slabs (one trip; tail of every length class), a batch,
    and a leading dimension beyond K."""
    for (M, N, ns, nb, pad) in [(520, 300, 24, 2, 0), (257, 513, 7, 1, 0), (300, 260, 11, 3, 1), (256, 256, 12, 1, 0)]:
        K = slabs(dtype, ns)
        ld = K + pad * 128 // gen.ELEM_BYTES[dtype]      # rows 128 bytes apart from tight
        inp = int_inputs(dtype, M, N, K, batch=nb, lda=ld, ldb=ld, seed=ns)
        q = run_exact(inp, "mfma32-direct-to-lds", flags=tile_flag)
        if bm:
            assert q.bm == bm


@pytest.mark.parametrize("dtype", [gen.BF16, gen.F16])
def test_both_matrix_instructions_of_the_256_tile_kernel_are_exact(dtype):
    """Two-byte types on 256-tiles multiply with v_mfma_f32_16x16x32 (8 x 8 accumulator tiles per wave; with 96 slabs
    or more the form that issues ahead of the slab barrier), or with v_mfma_f32_32x32x16 when the switch asks for it:
    edges in both directions, a bias, a two-byte output rounded to nearest even."""
    for (M, N, ns, nb, flag, suffix) in [(520, 300, 100, 1, 0, ""), (300, 520, 13, 2, 0, ""),
                                         (520, 300, 100, 1, gemm.GEMM_FLAG_MFMA_32X32, "-mfma32x32"),
                                         (300, 520, 13, 2, gemm.GEMM_FLAG_MFMA_32X32, "-mfma32x32")]:
        inp = int_inputs(dtype, M, N, slabs(dtype, ns), batch=nb, seed=ns + flag, biased=True)
        q = run_exact(inp, "mfma32-direct-to-lds" + suffix, flags=gemm.GEMM_FLAG_TILE_256 | flag)
        assert q.bm == 256
        C_ref, _ = oracle_for(inp)
        rc, _, raw = util.run_config(K4, inp, out_dtype=dtype, flags=gemm.GEMM_FLAG_TILE_256 | flag)
        assert rc == gemm.GEMM_OK
        want = gen.quantise(dtype, C_ref.astype(np.float32).reshape(-1))
        np.testing.assert_array_equal(raw.cpu().numpy().view(np.uint16)[: nb * M * N], want)


RING_CASES = [  # (M, N, slabs, batch): at least 256 tiles of 256 x 256, so the persistent kernel takes the product
    (520, 300, 3, 130),     # 780 tiles: workgroups with 3 and with 4 tiles; the shortest K the kernel takes (first, last-but-one, last slab)
    (520, 300, 4, 43),      # 258 tiles: one or two tiles per workgroup; one middle slab
    (256, 512, 11, 129),    # 258 interior tiles, middle-slab loop of 8
    (300, 260, 7, 70),      # 280 tiles, every one with an edge
]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("case", RING_CASES, ids=["%dx%dx%dslabs_b%d" % c for c in RING_CASES])
def test_persistent_kernel_is_exact(dtype, case):
    """The persistent form of the 256-tile kernel: the ring runs on across tile boundaries, so a wrong slab of
    the NEXT tile (stale region, wrong source, wrong wait) shows up in the tile after the boundary.  fp32
    output bit for bit against the oracle, and the two-byte output against the oracle's value rounded to
    nearest even (sums are integers: the kernel's fp32 accumulator holds them exactly before it rounds)."""
    M, N, ns, nb = case
    K = slabs(dtype, ns)
    inp = int_inputs(dtype, M, N, K, batch=nb, seed=ns, biased=(ns == 7))
    q = run_exact(inp, "mfma32-direct-to-lds(persistent)", flags=gemm.GEMM_FLAG_TILE_256)
    assert q.bm == 256 and q.grid == 256
    out = gen.BF16 if dtype == gen.E4M3 else dtype
    C_ref, _ = oracle_for(inp)
    rc, _, raw = util.run_config(K4, inp, out_dtype=out, flags=gemm.GEMM_FLAG_TILE_256)
    assert rc == gemm.GEMM_OK
    want = gen.quantise(out, C_ref.astype(np.float32).reshape(-1))
    got = raw.cpu().numpy().view(np.uint16)[: nb * M * N]
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("dtype", [gen.BF16, gen.F16])
@pytest.mark.parametrize("case", RING_CASES + [(1024, 768, 70, 22)], ids=["%dx%dx%dslabs_b%d" % c for c in RING_CASES + [(1024, 768, 70, 22)]])
def test_persistent_kernel_reads_a_row_major_b_in_place(dtype, case):
    """B stored row-major (N contiguous), aligned: the persistent kernel keeps B's slab in LDS as it lies in memory
    and reads the fragments with transposing LDS reads.  Integer operands, fp32 output: bit for bit.  The cases
    cover edge tiles (columns past N are whatever follows in memory and must only reach masked outputs), unequal
    tile counts per workgroup, a leading dimension beyond N, and a K of more than 64 slabs."""
    M, N, ns, nb = case
    K = slabs(dtype, ns)
    inp = int_inputs(dtype, M, N, K, ROW, ROW, batch=nb, ldb=N + (8 if ns == 7 else 0) + (-N) % 8, seed=ns + 100)
    q = run_exact(inp, "mfma32-direct-to-lds(persistent,B-row-major)", exact_path=False)    # (a thin remainder of rows may go to the thin kernel)
    assert q.grid == 256 and q.workspace_bytes == 0 and q.violated == 0


BROW_RAGGED = [  # (M, N, K, batch, lda - K, ldb - N, path suffix)
    (520, 300, 256, 43, 1, 1, ""),             # odd leading dimensions: every row aligned to an element only
    (512, 509, 320, 70, 3, 0, ""),             # N odd: the last row of B ends in the middle of a dword
    (512, 509, 321, 70, 0, 0, ""),             # K odd as well: a last slab of one element, A's last row ends mid-dword
    (700, 515, 203, 29, 0, 0, ""),             # three whole slabs and a ragged fourth, edge tiles in both directions
    (4099, 4093, 449, 1, 0, 0, "+thin(M-tail)"),   # the ragged fp16 workload's shape with a shorter K: 16 x 16 tiles, 3 rows to the thin kernel
    (4096 + 40, 4096, 200, 1, 0, 5, "+thin(M-tail)"),  # 40 rows: four row groups in the thin kernel
    (4096 + 17, 4093, 203, 1, 1, 1, "+thin(M-tail)"),  # 17 rows: two row groups, odd leading dimensions
    (1024 + 64, 1000, 333, 64, 0, 3, "+thin(M-tail)"), # batched: 4 x 4 tiles x 64 = 4 rounds, the fifth row of tiles would be a fifth
    (4096 + 65, 4096, 200, 1, 0, 0, ""),               # 65 rows stay a row of tiles
]


@pytest.mark.parametrize("dtype", [gen.BF16, gen.F16])
@pytest.mark.parametrize("case", BROW_RAGGED, ids=["%dx%dx%d_b%d_%d_%d%s" % c for c in BROW_RAGGED])
def test_row_major_operands_with_odd_leading_dimensions_and_ragged_k_in_place(dtype, case):
    """A and B row-major, nothing aligned, K not whole slabs, no scratch lent: the persistent kernel loads the rows
    with under-aligned 16-byte loads, clears what lies beyond K in the last slab (the gaps between rows hold 3, the
    operands' neighbours whatever the allocator left); a thin remainder of rows that would cost a round of tiles is
    multiplied by the thin kernel, which reads B in place as well."""
    M, N, K, nb, pa, pb, suffix = case
    inp = int_inputs(dtype, M, N, K, ROW, ROW, batch=nb, lda=K + pa, ldb=N + pb, seed=K)
    q = run_exact(inp, "mfma32-direct-to-lds(persistent,B-row-major)" + suffix)
    assert q.violated == 0


THIN_CASES = [  # (M, N, K, batch, lda - K, ldb - N, biased)
    (1, 64, 32, 1, 0, 0, False),               # one row, one strip, one k tile: seven of the eight waves have nothing
    (3, 4093, 4097, 1, 0, 0, False),           # the ragged workload's remainder as a product of its own
    (16, 1000, 777, 1, 1, 1, True),            # one full row group, odd leading dimensions, bias
    (17, 130, 2050, 3, 3, 0, False),           # two row groups, batched, a strip of two columns
    (32, 515, 256, 2, 0, 5, False),
    (33, 257, 1031, 1, 0, 0, True),            # four row groups (two sets of registers), one-column last strip
    (64, 2048, 1024, 1, 0, 0, False),          # everything whole and aligned
    (64, 777, 95, 2, 5, 1, False),             # fewer k tiles than waves x sets
    # many strips
    (5, 8200, 100, 1, 0, 0, False),
    (20, 4100, 203, 2, 1, 1, True),            # two row groups, batched
    (40, 1030, 300, 8, 0, 3, False),           # four row groups (two sets of registers)
]


@pytest.mark.parametrize("dtype", [gen.BF16, gen.F16])
@pytest.mark.parametrize("case", THIN_CASES, ids=["%dx%dx%d_b%d_%d_%d_%s" % c for c in THIN_CASES])
def test_thin_kernel_reads_a_row_major_b_in_place(dtype, case):
    """At most 64 rows, A and B row-major, nothing aligned, any K, no scratch: a strip of 64 columns per workgroup,
    K dealt to its eight waves, B parked as it lies in memory and read back with transposing LDS reads.  fp32 output
    bit for bit, and the two-byte output against the oracle's value rounded to nearest even."""
    M, N, K, nb, pa, pb, biased = case
    inp = int_inputs(dtype, M, N, K, ROW, ROW, batch=nb, lda=K + pa, ldb=N + pb, seed=K + M, biased=biased)
    q = run_exact(inp, "mfma16-thin(B-row-major)")
    cols = 64
    assert q.violated == 0 and q.workspace_bytes == 0 and q.grid == -(-N // cols) * nb and q.bn == cols
    C_ref, _ = oracle_for(inp)
    rc, _, raw = util.run_config(K4, inp, out_dtype=dtype)
    assert rc == gemm.GEMM_OK
    want = gen.quantise(dtype, C_ref.astype(np.float32).reshape(-1))
    got = raw.cpu().numpy().view(np.uint16)[: nb * M * N]
    np.testing.assert_array_equal(got, want)


def at_page_end(arr, at_end):
    """The array's bytes on the GPU, ending with a 4 KiB page when `at_end` (the page after belongs to the same allocation)."""
    raw = np.ascontiguousarray(arr).view(np.uint8)
    buf = torch.empty(raw.size + 2 * 4096, dtype=torch.uint8, device="cuda")
    lead = (-(buf.data_ptr() + raw.size)) % 4096 if at_end else 256
    assert lead % 2 == 0
    d = buf[lead: lead + raw.size]
    d.copy_(torch.from_numpy(raw.copy()))
    assert ((d.data_ptr() + raw.size) % 4096 == 0) == at_end
    return d


@pytest.mark.parametrize("dtype", [gen.BF16, gen.F16])
@pytest.mark.parametrize("a_end,b_end,suffix", [(True, False, "+thin(last row)"), (False, True, "+masked(last col)"),
                                                (True, True, "+split(row,col)")])
def test_row_major_b_with_an_operand_ending_at_the_end_of_a_page(dtype, a_end, b_end, suffix):
    """K and N odd and an operand's last byte the last of a 4 KiB page: the element after it, which the persistent
    kernel's loads of the operand's last row touch, may not be mapped.  A's last row then goes to the thin kernel, C's
    last column (B's last element of every row) to the masked kernel, and the rest stays in place."""
    M, N, K, nb = 520, 2101, 301, 15                    # 3 x 9 tiles x 15 >= 256, also without the last column
    inp = int_inputs(dtype, M, N, K, ROW, ROW, batch=nb, seed=5, biased=True)
    dA, dB = at_page_end(inp.A, a_end), at_page_end(inp.B, b_end)
    d = gemm.make_desc(M, N, K, dtype, gen.F32, ROW, ROW, lda=inp.lda, ldb=inp.ldb, ldc=inp.ldc, batch=nb, stride_a=inp.stride_a,
                       stride_b=inp.stride_b, stride_c=inp.stride_c)
    assert gemm.gemm_query(K4, d).path == "mfma32-direct-to-lds(persistent,B-row-major)"            # (no addresses: nothing known)
    q = gemm.gemm_query(K4, d, dA, dB)
    assert q.path == "mfma32-direct-to-lds(persistent,B-row-major)" + suffix and q.violated == 0, q.path
    C_ref, _ = oracle_for(inp)
    rc, C, _ = util.run_config(K4, inp, dA=dA, dB=dB)
    assert rc == gemm.GEMM_OK, gemm.gemm_status_string(rc)
    np.testing.assert_array_equal(C[:, :, :N], C_ref)


OFF_DWORD_CASES = [  # (M, N, K, batch, lda, ldb, extra batch stride of A, of B, A's address off by an element, B's)
    (3, 200, 300, 1, 300, 200, 0, 0, True, False),     # even rows throughout, A starts 2 bytes off a dword
    (16, 129, 130, 1, 130, 130, 0, 0, False, True),    # ... B does
    (33, 257, 515, 1, 516, 258, 0, 0, True, True),     # ... both do (four row groups)
    (20, 70, 1000, 3, 1000, 70, 1, 0, False, False),   # even rows, A's batch items an odd number of elements apart
    (64, 100, 96, 4, 96, 100, 0, 1, False, False),     # ... B's
    (7, 333, 1025, 2, 1025, 333, 1, 1, True, True),    # odd rows, odd batch strides, both addresses off
    (48, 4097, 65, 1, 65, 4097, 0, 0, True, False),    # odd rows and A off: even rows of A are the aligned ones
]


@pytest.mark.parametrize("dtype", [gen.BF16, gen.F16])
@pytest.mark.parametrize("case", OFF_DWORD_CASES, ids=["%dx%dx%d_b%d_ld%d_%d_s%d_%d_%s_%s" % c for c in OFF_DWORD_CASES])
def test_thin_kernel_realigns_rows_that_start_two_bytes_off_a_dword(dtype, case):
    """Rows of A that start on an odd element are loaded as whole aligned dwords and shifted into place in registers
    (B's are loaded where they lie): the start of an operand, an odd batch stride and an odd leading dimension each
    put rows 2 bytes off a dword.  The elements before the first and after the last one of each operand hold 3 (as
    the gaps between rows do): a kernel that let them into a sum would be off by an integer."""
    M, N, K, nb, lda, ldb, xa, xb, off_a, off_b = case
    inp = int_inputs(dtype, M, N, K, ROW, ROW, batch=nb, lda=lda, ldb=ldb, seed=M + K)
    sa, sb = M * lda + xa, K * ldb + xb
    three = gen.quantise(dtype, np.full(1, 3.0, dtype=np.float32))[0]

    def spread(x, per_item, stride, lead):            # batch items `stride` apart behind `lead` elements, 3 elsewhere
        out = np.full(lead + nb * stride + 8, three, dtype=x.dtype)
        for b in range(nb):
            out[lead + b * stride: lead + b * stride + per_item] = x[b * per_item: (b + 1) * per_item]
        return out
    A, B = spread(inp.A, M * lda, sa, int(off_a)), spread(inp.B, K * ldb, sb, int(off_b))
    dA, dB = util.dev(A), util.dev(B)
    dA, dB = dA[2 * int(off_a):], dB[2 * int(off_b):]
    assert dA.data_ptr() % 4 == 2 * int(off_a) and dB.data_ptr() % 4 == 2 * int(off_b)
    moved = gen.Inputs(inp.cfg, inp.seed, A[int(off_a):], B[int(off_b):], lda, ldb, inp.ldc, sa, sb, inp.stride_c)
    d = gemm.make_desc(M, N, K, dtype, gen.F32, ROW, ROW, lda=lda, ldb=ldb, ldc=inp.ldc, batch=nb, stride_a=sa, stride_b=sb,
                       stride_c=inp.stride_c)
    assert gemm.gemm_query(K4, d, dA, dB).path == "mfma16-thin(B-row-major)"
    C_ref, _ = oracle_for(moved)
    rc, C, _ = util.run_config(K4, moved, dA=dA, dB=dB)
    assert rc == gemm.GEMM_OK, gemm.gemm_status_string(rc)
    np.testing.assert_array_equal(C[:, :, :N], C_ref)


@pytest.mark.parametrize("dtype", DTYPES)
def test_nine_region_ring_of_the_small_tile_kernel_is_exact(dtype):
    """128-tiles that number at most one per CU, K of 32 slabs or more: prefetch 3.5 slabs deep.  33 slabs: first slab,
    three trips of the nine-slab loop, five slabs of tail; 45: four trips and eight; 32: the fewest.  M and N end
    inside a tile; a batch; a leading dimension beyond K; and the same kernel under split-K's K ranges."""
    for (M, N, ns, nb, pad, tile) in [(520, 300, 33, 2, 0, gemm.GEMM_FLAG_TILE_128), (257, 513, 45, 1, 8, gemm.GEMM_FLAG_TILE_128),
                                      (1000, 900, 32, 1, 0, 0), (128, 128, 40, 3, 0, gemm.GEMM_FLAG_TILE_128)]:
        K = slabs(dtype, ns)
        inp = int_inputs(dtype, M, N, K, batch=nb, lda=K + pad * 16 // gen.ELEM_BYTES[dtype], seed=ns)
        q = run_exact(inp, "mfma32-direct-to-lds", flags=tile)
        assert (q.bm, q.stages, q.lds_bytes) == (128, 4, 9 * 128 * 128), (q.bm, q.stages, q.lds_bytes)
    # 31 slabs, or more than 256 tiles: the five-region ring
    for (M, N, ns, nb) in [(520, 300, 31, 2), (2100, 2100, 33, 1)]:
        inp = int_inputs(dtype, M, N, slabs(dtype, ns), batch=nb, seed=ns)
        q = run_exact(inp, "mfma32-direct-to-lds", flags=gemm.GEMM_FLAG_TILE_128)
        assert (q.bm, q.stages, q.lds_bytes) == (128, 2, 5 * 128 * 128)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("flags,tag", [(gemm.GEMM_FLAG_DEOPT_NO_SWIZZLE, "-noswz"), (gemm.GEMM_FLAG_DEOPT_NO_OVERLAP, "-noovl"),
                                       (gemm.GEMM_FLAG_DEOPT_NO_RASTER, "-noraster"),
                                       (gemm.GEMM_FLAG_DEOPT_NO_RASTER | gemm.GEMM_FLAG_TILE_128, "-noraster")])
def test_simplified_expert_states_are_exact(dtype, flags, tag):
    inp = int_inputs(dtype, 520, 300, slabs(dtype, 17), batch=2, seed=3)
    run_exact(inp, "mfma32-direct-to-lds" + tag, flags=flags)


@pytest.mark.parametrize("dtype", DTYPES)
def test_split_k_form_is_exact(dtype):
    """Few tiles, long K, scratch lent: K ranges as batch items of the fast kernel, then the adding pass."""
    for (M, N, ns, kw) in [(100, 300, 64, dict(biased=True)), (200, 257, 32, {}), (64, 1024, 128, dict(ldc=1032))]:
        inp = int_inputs(dtype, M, N, slabs(dtype, ns), seed=ns, **kw)
        run_exact(inp, "+splitK(", lend=True, exact_path=False)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("la,lb,path", [(ROW, ROW, "mfma32-packed+direct-to-lds"), (COL, ROW, "mfma32-packed+direct-to-lds"),
                                        (COL, COL, "mfma32-packed+direct-to-lds"), (ROW, COL, "mfma32-packed+direct-to-lds")])
def test_packed_path_is_exact(dtype, la, lb, path):
    """Odd leading dimensions and a ragged K in every layout pair, scratch lent: both pack kernels (rows
    and transposing), zero padding of K, then the fast kernel on the copies."""
    M, N, K = 300, 270, 1203
    inp = int_inputs(dtype, M, N, K, la, lb, batch=2, lda=(K if la == ROW else M) + 3, ldb=(N if lb == ROW else K) + 5,
                     ldc=N + 1, seed=7)
    run_exact(inp, path, lend=True)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("la,lb,tag", [(ROW, ROW, "(B)"), (COL, COL, "(A)")])
def test_packed_path_with_one_operand_in_place_is_exact(dtype, la, lb, tag):
    inp = int_inputs(dtype, 392, 264, slabs(dtype, 9), la, lb, batch=2, seed=8)
    run_exact(inp, "mfma32-packed%s+direct-to-lds" % tag, lend=True)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("rem", [3, 17, 48, 64])
def test_row_remainder_split_is_exact(dtype, rem):
    """16 rows of 256-tiles by 16 columns plus a thin remainder: the tiled kernel and the streaming kernel
    (one, two, three, four groups of rows) each write their part of one C."""
    inp = int_inputs(dtype, 4096 + rem, 4096, slabs(dtype, 8), seed=rem)
    run_exact(inp, "mfma32-direct-to-lds(persistent)+stream(M-tail)")      # 256 whole tiles of 8 slabs: the persistent form


STREAM_CASES = [  # (M, N, K in 2-byte units, batch, what)
    (16, 8200, 1032, 1, "16 rows, one wave per strip of 16 columns"),
    (9, 1000, 2056, 1, "16 rows, K tiles dealt to 4 waves"),
    (32, 4100, 1032, 1, "two groups of rows"),
    (47, 8200, 520, 1, "three groups"),
    (64, 8200, 520, 1, "four groups"),
    (96, 8200, 520, 1, "six groups"),
    (81, 530, 1160, 16, "six groups, batched"),
]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("case", STREAM_CASES, ids=[c[4] for c in STREAM_CASES])
def test_streaming_kernel_is_exact(dtype, case):
    """Every form of the streaming kernel, with ragged row groups, a ragged last strip and a ragged last K
    tile (K a multiple of 16 bytes only)."""
    M, N, K2, nb, _ = case
    K = K2 * 2 // gen.ELEM_BYTES[dtype]
    q = run_exact(int_inputs(dtype, M, N, K, batch=nb, seed=M), "mfma16-stream(small-M)")
    assert q.bm == (16 * ((M + 15) // 16) if M <= 64 else 96)


@pytest.mark.parametrize("dtype", DTYPES)
def test_streaming_kernel_forms_forced_by_the_sweep_flags_are_exact(dtype):
    """GEMM_FLAG_STREAM_FORM: every compiled form that holds the product's rows, on 9 rows (all six) and on 40 rows
    (the three forms of 48, 64 and 96 rows), and on the transposed (few columns) product."""
    eb = gen.ELEM_BYTES[dtype]
    for (M, N, K2, forms) in [(9, 1000, 1032, range(6)), (40, 8200, 520, (3, 4, 5)), (4100, 7, 136, range(6))]:
        inp = int_inputs(dtype, M, N, K2 * 2 // eb, seed=M)
        for f in forms:
            run_exact(inp, "-form%d" % f, flags=gemm.GEMM_FLAG_STREAM_FORM(f), exact_path=False)
    # a form with fewer rows than the product, or the override on a product that does not stream, is refused
    d = gemm.make_desc(40, 8200, 1024, dtype, gen.F32, ROW, COL, flags=gemm.GEMM_FLAG_STREAM_FORM(2))
    assert gemm.gemm_query(K4, d).status == gemm.GEMM_ERR_BAD_ARG
    d = gemm.make_desc(512, 512, 1024, dtype, gen.F32, ROW, COL, flags=gemm.GEMM_FLAG_STREAM_FORM(0))
    assert gemm.gemm_query(K4, d).status == gemm.GEMM_ERR_BAD_ARG


@pytest.mark.parametrize("dtype", DTYPES)
def test_one_tile_per_workgroup_form_forced_on_a_product_the_persistent_kernel_would_take(dtype):
    inp = int_inputs(dtype, 520, 300, slabs(dtype, 5), batch=43, seed=5)
    q = run_exact(inp, "mfma32-direct-to-lds-nopersist", flags=gemm.GEMM_FLAG_TILE_256 | gemm.GEMM_FLAG_DEOPT_NO_PERSISTENT)
    assert q.grid == 6 * 43


@pytest.mark.parametrize("dtype", DTYPES)
def test_streaming_kernel_on_few_columns_is_exact(dtype):
    for (M, N, K2) in [(4100, 7, 136), (8200, 33, 264), (8200, 80, 392)]:
        K = K2 * 2 // gen.ELEM_BYTES[dtype]
        run_exact(int_inputs(dtype, M, N, K, seed=N, biased=True), "mfma16-stream(small-N)")


@pytest.mark.parametrize("dtype", DTYPES + [gen.F32])
def test_masked_kernel_is_exact(dtype):
    """No scratch, ragged K, odd leading dimensions: the masked kernel in both of its tile sizes."""
    for (M, N, K) in [(259, 130, 1000), (1100, 2100, 203)]:
        inp = int_inputs(dtype, M, N, K, ROW, ROW, lda=K + 1, ldb=N + 3, seed=K)
        run_exact(inp, "masked", exact_path=False)


def test_headline_shape_full_size_is_exact():
    """bf16 8192^3, A row-major, B column-major, fp32 out, integer-valued operands: all 67 million outputs
    of the launch configuration the benchmark times (256-tiles, 1024 workgroups, 128 slabs each) against
    the oracle's full product.  Partial sums stay below 4 * 8192 < 2^24."""
    M = N = K = 8192
    rng = np.random.default_rng(8192)
    A = gen.quantise(gen.BF16, rng.integers(-2, 3, M * K).astype(np.float32))
    B = gen.quantise(gen.BF16, rng.integers(-2, 3, N * K).astype(np.float32))
    cfg = gen.Config("C2_ints", M, N, K, gen.BF16, gen.F32, ROW, COL, "uniform")
    inp = gen.Inputs(cfg, 0, A, B, K, K, N, M * K, N * K, M * N)
    d = gemm.make_desc(M, N, K, gen.BF16, gen.F32, ROW, COL)
    q = gemm.gemm_query(K4, d)
    assert q.path == "mfma32-direct-to-lds" and q.bm == 256 and q.grid == 1024
    C_ref, _ = oracle_for(inp)
    rc, C, _ = util.run_config(K4, inp)
    assert rc == gemm.GEMM_OK
    C = C.reshape(M, N)
    bad = np.flatnonzero(C != C_ref[0])
    assert bad.size == 0, f"{bad.size} outputs differ, first at {np.unravel_index(bad[0], (M, N))}"
    torch.cuda.empty_cache()
