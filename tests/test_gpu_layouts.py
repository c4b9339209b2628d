"""Layout converters of the library against the layout formulas written out in numpy:
byte-exact."""
import numpy as np
import pytest
import torch

import layouts
from gpu_util import DEV, to_dev, tdtype
from paper_2406_17404_amd import binding as b

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("kind,n_out,n_in,H,dh", [
    ("plain", 96, 48, 0, 0), ("gate_up", 128, 64, 0, 0), ("qkv", 3 * 2 * 64, 32, 2, 64),
    ("qkv", 3 * 3 * 128, 80, 3, 128), ("plain", 4096, 1024, 0, 0),
    ("qkv", (8 + 2 * 2) * 64, 48, 8, 64), ("qkv", (4 + 2 * 1) * 128, 32, 4, 128)])   # grouped-query
def test_pack_weight(dtype, kind, n_out, n_in, H, dh):
    rng = np.random.default_rng(0)
    w = rng.integers(-100, 100, size=(n_out, n_in)).astype(np.float32)  # exact in bf16
    want = layouts.pack_weight(w, kind, H, dh)
    src = to_dev(w, tdtype(dtype))
    dst = torch.empty_like(src)
    code = {"plain": b.PACK_PLAIN, "qkv": b.PACK_QKV, "gate_up": b.PACK_GATE_UP}[kind]
    b.trj_pack_weight(dst, src, n_out, n_in, b.BF16 if dtype == "bf16" else b.F32, code, H, dh)
    assert np.array_equal(dst.float().cpu().numpy().ravel(), want)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("H,dh,s_pool,slot0,n", [(2, 64, 64, 0, 64), (3, 128, 160, 37, 101),
                                                 (1, 32, 32, 5, 0), (1, 96, 96, 1, 95)])
def test_kv_pack_unpack(dtype, H, dh, s_pool, slot0, n):
    rng = np.random.default_rng(1)
    k = rng.integers(-120, 120, size=(H, n, dh)).astype(np.float32)
    v = rng.integers(-120, 120, size=(H, n, dh)).astype(np.float32)
    dt, code = tdtype(dtype), (b.BF16 if dtype == "bf16" else b.F32)
    kp = torch.zeros(H, s_pool * dh, dtype=dt, device=DEV)
    vp = torch.zeros_like(kp)
    b.trj_kv_pack(kp, vp, to_dev(k, dt), to_dev(v, dt), H, dh, s_pool, slot0, n, code)
    wk, wv = layouts.kv_to_pool(k, v, s_pool, slot0)
    assert np.array_equal(kp.float().cpu().numpy(), wk)
    assert np.array_equal(vp.float().cpu().numpy(), wv)
    k2 = torch.empty(H, n, dh, dtype=dt, device=DEV)
    v2 = torch.empty_like(k2)
    b.trj_kv_unpack(k2, v2, kp, vp, H, dh, s_pool, slot0, n, code)
    assert np.array_equal(k2.float().cpu().numpy(), k) and np.array_equal(v2.float().cpu().numpy(), v)
