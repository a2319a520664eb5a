"""GPU parity at the full benchmark sizes, in the launch configuration the benchmark times.

The oracle evaluates sampled outputs one by one (random points, whole boundary rows and columns,
points around workgroup-tile corners) instead of the full product; C1 is small enough to be
checked completely in the other parity file.  Seeds 0..2 for the expert variant (three seeds, as
the gate prescribes), seed 0 for the earlier lineage states to keep the run short.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_28213_amd import gemm
from paper_2605_28213_amd import inputs as gen
from tests import util

pytestmark = pytest.mark.gpu


def sample_points(cfg, rng, n_random=3000):
    M, N, nb = cfg.M, cfg.N, cfg.batch
    pb = [rng.integers(0, nb, n_random)]
    pi = [rng.integers(0, M, n_random)]
    pj = [rng.integers(0, N, n_random)]
    # last row / last column / first row of a random batch item: where tails and masks live
    b = int(rng.integers(0, nb))
    cols = rng.choice(N, size=min(N, 1024), replace=False)
    rows = rng.choice(M, size=min(M, 1024), replace=False)
    for i in (0, M - 1):
        pb.append(np.full(cols.size, b)); pi.append(np.full(cols.size, i)); pj.append(cols)
    for j in (0, N - 1):
        pb.append(np.full(rows.size, b)); pi.append(rows); pj.append(np.full(rows.size, j))
    # corners of 256 x 256 tiles
    ti = np.array([t for t in (255, 256, 257, 2047, 2048, 4095, 4096) if t < M])
    tj = np.array([t for t in (255, 256, 257, 2047, 2048, 4095, 4096) if t < N])
    if ti.size and tj.size:
        gi, gj = np.meshgrid(ti, tj, indexing="ij")
        pb.append(np.full(gi.size, b)); pi.append(gi.ravel()); pj.append(gj.ravel())
    return np.concatenate(pb), np.concatenate(pi), np.concatenate(pj)


def run_full(name, seed, variants):
    cfg = gen.CONFIGS[name]
    inp = gen.make_inputs(cfg, seed)
    rng = np.random.default_rng(100 + seed)
    pb, pi, pj = sample_points(cfg, rng)
    C_ref, D = oracle.gemm_points(cfg.in_dtype, cfg.layout_a, cfg.layout_b, cfg.M, cfg.N, cfg.K, inp.A, inp.lda,
                                  inp.B, inp.ldb, pb, pi, pj, batch=cfg.batch, stride_a=inp.stride_a,
                                  stride_b=inp.stride_b, scale_a=inp.scale_a, scale_b=inp.scale_b)
    dA, dB = util.dev(inp.A), util.dev(inp.B)
    for v in variants:
        print(f"[full-size] {name} seed {seed} {gemm.gemm_variant_name(v)}", flush=True)
        rc, C, _ = util.run_config(v, inp, dA=dA, dB=dB)
        assert rc == gemm.GEMM_OK
        assert np.all(np.isfinite(C[:, :, : cfg.N]))
        err = util.norm_err(C[pb, pi, pj], C_ref, D)
        assert err <= util.TOL[cfg.in_dtype], f"{gemm.gemm_variant_name(v)} on {name} seed {seed}: {err:.3e}"
    del dA, dB
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name", ["C2", "C3", "C4", "C5"])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_expert_variant_full_size(name, seed):
    run_full(name, seed, [gemm.GEMM_K4_MFMA])


@pytest.mark.parametrize("name", ["C2", "C3", "C4", "C5"])
def test_earlier_lineage_states_full_size(name):
    run_full(name, 0, [gemm.GEMM_K0_NAIVE, gemm.GEMM_K1_LDS_TILED, gemm.GEMM_K2_VECTORIZED, gemm.GEMM_K3_PIPELINED])
