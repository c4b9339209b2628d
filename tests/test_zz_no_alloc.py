"""tree_attention_static_scratch (the entry point for callers that cannot allocate: its
scratch is a fixed array inside the library) against tree_attention on the same inputs:
two calls in a row on one stream, the second with a smaller input, so that whatever the
first call left in the shared array must not leak into the second."""
import numpy as np
import pytest
import torch

import layouts
from gpu_util import DEV, Batch, rel_err, to_dev
from oracle import tr_oracle as O
from paper_2406_17404_amd import binding as b
from paper_2406_17404_amd import inputs as I

pytestmark = pytest.mark.gpu


def case(seed, H, dh, L, N, dtype):
    q, k, v, parent = I.gen_attention_case(seed, H, dh, L, N, dtype)
    batch = Batch([parent], [L])
    kp = np.full((H, batch.s_pool * dh), np.nan, np.float32)
    vp = np.full((H, batch.s_pool * dh), np.nan, np.float32)
    layouts.kv_to_pool(k, v, batch.s_pool, 0, kp, vp)
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    return dict(q=q, k=k, v=v, parent=parent, batch=batch, L=L, N=N, H=H, dh=dh, dt=dt,
                code=b.BF16 if dtype == "bf16" else b.F32,
                dq=to_dev(q, dt), dk=to_dev(kp, dt), dv=to_dev(vp, dt))


def call(c, static):
    bt, N, H, dh = c["batch"], c["N"], c["H"], c["dh"]
    out = torch.full((N, H, dh), float("nan"), dtype=c["dt"], device=DEV)
    args = (c["dq"], c["dk"], c["dv"], bt.parent, bt.node_off, bt.kv_off, bt.prefix, 1, N, H, dh,
            bt.s_pool, c["L"] + N, c["code"], float(1 / np.sqrt(dh)))
    if static:
        b.tree_attention_static_scratch(*args, out)
    else:
        desc = b.ModelDesc(1, 64, H, dh, 64, 64, 1e-5, 1e4, c["code"])
        ws = torch.empty(b.trj_workspace_bytes(desc, N, 1, c["L"] + N), dtype=torch.uint8, device=DEV)
        b.tree_attention(*args, ws, out)
    return out


@pytest.mark.parametrize("dtype,tol", [("bf16", 1e-2), ("f32", 1e-5)])
def test_static_scratch_equals_workspace_entry_point(dtype, tol):
    # bf16: the first call splits the keys over several workgroups per head (partials and
    # their merge live in the scratch array), the second is a small single-tile case
    big = case(501, 32, 128, 2048, 64, dtype) if dtype == "bf16" else case(501, 4, 64, 700, 64, dtype)
    small = case(502, 8, 128, 300, 20, dtype) if dtype == "bf16" else case(502, 4, 64, 90, 9, dtype)
    got_big = call(big, True)        # two calls in a row on one stream, nothing in between
    got_small = call(small, True)
    torch.cuda.synchronize()
    for c, got in ((big, got_big), (small, got_small)):
        ref = call(c, False)
        torch.cuda.synchronize()
        g, r = got.float().cpu().numpy(), ref.float().cpu().numpy()
        assert np.isfinite(g).all()
        assert np.array_equal(g, r)          # same kernels, same launch plan: the same bits
        heads = [0, c["H"] - 1]
        want = O.tree_attention(c["q"][:, heads], c["k"][heads], c["v"][heads], c["parent"], c["L"])
        assert rel_err(g[:, heads], want) <= tol


def test_static_scratch_rejects_what_does_not_fit_and_touches_nothing():
    # with the launch knob asking for 4096 workgroups a 64k-slot sequence is split 128 ways
    # and its partial sums alone exceed the array
    N, H, dh, L = 64, 32, 128, 65536
    out = torch.full((64,), 5.0, dtype=torch.bfloat16, device=DEV)
    t = torch.zeros(1024, dtype=torch.int32, device=DEV)
    b.trj_set_tunable("attn_target_wgs", 4096)
    try:
        need = b.tree_attention_workspace_bytes(1, N, H, dh, L + N, b.BF16)
        assert need > b.STATIC_SCRATCH_BYTES, need
        with pytest.raises(b.TrjError) as e:
            b.tree_attention_static_scratch(t, t, t, t, t, t, t, 1, N, H, dh, (L + N + 31) // 32 * 32,
                                            L + N, b.BF16, 0.1, out)
        assert e.value.status == -5
    finally:
        b.trj_set_tunable("attn_target_wgs", 256)
    torch.cuda.synchronize()
    assert bool((out == 5.0).all())
    assert b.tree_attention_workspace_bytes(1, N, H, dh, L + N, b.BF16) <= b.STATIC_SCRATCH_BYTES
