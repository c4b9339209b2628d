"""The development aids of include/trjacobi_dev.h that the benchmark relies on: the copy
kernel copies exactly, the read kernel leaves its sink alone, the device reports itself,
and the launch-plan query names the kernels the workloads are documented to run."""
import pytest
import torch

from paper_2406_17404_amd import binding as b

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_copy_and_read_probes():
    n = 1 << 24
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device=DEV)
    dst = torch.zeros_like(src)
    b.trj_copy_probe(dst, src, n)
    sink = torch.zeros(1, dtype=torch.int32, device=DEV)
    b.trj_read_probe(src, n, sink)
    torch.cuda.synchronize()
    assert torch.equal(dst, src) and int(sink.cpu()) == 0
    with pytest.raises(b.TrjError):
        b.trj_copy_probe(dst, src, 24)          # not a multiple of 16


def test_device_reports_itself():
    info = b.trj_dev_device_info()
    assert info["compute_units"] >= 1 and info["clock_khz"] > 0 and info["memory_bus_bits"] > 0
    assert info["lds_bytes_per_workgroup"] >= 64 * 1024


def test_launch_plans_of_the_documented_workloads():
    d, F = 4096, 11008
    gu64 = b.trj_dev_gemm_plan(64, d, 2 * F, True)     # 64 rows: three row tiles, two k-parts
    assert (gu64["token_tiles"], gu64["row_tiles"], gu64["k_parts"], gu64["many_rows"]) == (2, 3, 2, 0)
    o64 = b.trj_dev_gemm_plan(64, d, d, False)         # split-k projection: 8 ways up to 64 rows
    assert o64["split_k"] == 8 and o64["many_rows"] == 0
    lm = b.trj_dev_gemm_plan(64, d, 32000, True)
    assert (lm["row_tiles"], lm["k_parts"]) == (4, 1)
    assert b.trj_dev_gemm_plan(1024, d, 2 * F, True)["many_rows"] == 1
