"""The projection kernel alone (trj_linear) against a plain fp64 matrix product."""
import numpy as np
import pytest
import torch

from gpu_util import DEV, rel_err, tdtype, to_dev
from paper_2406_17404_amd import binding as b
from paper_2406_17404_amd import inputs as I

pytestmark = pytest.mark.gpu


def run_linear(dtype, T, n_in, n_out, split_k, seed=0):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, n_in)).astype(np.float32)
    w = (rng.standard_normal((n_out, n_in)) * 0.05).astype(np.float32)
    if dtype == "bf16":
        x, w = I.bf16_round(x), I.bf16_round(w)
    dt, code = tdtype(dtype), (b.BF16 if dtype == "bf16" else b.F32)
    wd = to_dev(w, dt)
    wp = torch.empty_like(wd)
    b.trj_pack_weight(wp, wd, n_out, n_in, code, b.PACK_PLAIN)
    y = torch.full((T, n_out), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(2 * 128 * ((T + 127) // 128) * n_in + 32 * T * n_out + 1024, dtype=torch.uint8, device=DEV)
    b.trj_linear(to_dev(x, dt), wp, T, n_in, n_out, code, split_k, ws, y)
    torch.cuda.synchronize()
    return y.cpu().numpy(), x.astype(np.float64) @ w.astype(np.float64).T


@pytest.mark.parametrize("T,n_in,n_out,split_k", [
    (1, 16, 32, 0), (15, 256, 96, 0), (64, 4096, 512, 1), (64, 4096, 512, 4), (33, 1040, 160, 3),
    (128, 688, 96, 0), (100, 2048, 256, 2), (200, 512, 64, 0), (64, 11008, 128, 8),
    # 65..96 rows: three row tiles per pass (every workgroup shape the plan picks there)
    (69, 4096, 512, 0), (96, 1040, 160, 3), (80, 2064, 4128, 1), (65, 11008, 256, 4), (90, 4096, 6144, 1),
    # many rows: the kernel whose wavefronts own two row tiles (ragged row-tile count, split-k,
    # a k-range that ends inside a phase, rows that are not a multiple of 128)
    (256, 1024, 4096, 0), (512, 2064, 4128, 0), (1000, 512, 8192, 3), (1024, 4096, 2080, 2),
    (300, 1024, 2048, 0)])
def test_bf16_linear(T, n_in, n_out, split_k):
    got, want = run_linear("bf16", T, n_in, n_out, split_k)
    assert np.isfinite(got).all()
    # bf16 inputs are exact on both sides, products are exact in fp32: only the fp32
    # accumulation order differs
    assert rel_err(got, want) <= 1e-5


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5, 6])
@pytest.mark.parametrize("T,n_in,n_out,split_k", [(64, 1040, 160, 1), (33, 4096, 6144, 1), (128, 2064, 96, 3),
                                                  (20, 528, 416, 2), (69, 1040, 224, 2)])
def test_bf16_linear_every_workgroup_shape(cfg, T, n_in, n_out, split_k):
    """Row tiles x k-parts per workgroup forced to each of the six shapes (row-tile counts
    that do not divide by the shape's rows, a k-range that ends inside a phase)."""
    try:
        b.trj_set_tunable("gemm_cfg", cfg)
        got, want = run_linear("bf16", T, n_in, n_out, split_k)
    finally:
        b.trj_set_tunable("gemm_cfg", 0)
    assert np.isfinite(got).all()
    assert rel_err(got, want) <= 1e-5


@pytest.mark.parametrize("T,n_in,n_out,wt", [
    (1024, 528, 4128, 4),    # 129 row tiles: the last workgroup of 16 holds one
    (512, 2064, 8192, 4), (300, 1024, 6176, 4), (512, 2064, 8192, 2),
    (1024, 256, 16384, 0)])  # 0: the plan itself picks four row tiles per wavefront here
def test_bf16_linear_many_rows_tiles_per_wavefront(T, n_in, n_out, wt):
    try:
        b.trj_set_tunable("gemm_big_wt", wt)
        got, want = run_linear("bf16", T, n_in, n_out, 1)
    finally:
        b.trj_set_tunable("gemm_big_wt", 0)
    assert np.isfinite(got).all()
    assert rel_err(got, want) <= 1e-5


@pytest.mark.parametrize("T,n_in,n_out", [(15, 256, 768), (3, 1024, 64), (64, 48, 2048)])
def test_f32_linear(T, n_in, n_out):
    got, want = run_linear("f32", T, n_in, n_out, 0)
    assert rel_err(got, want) <= 1e-5
