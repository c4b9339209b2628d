"""The static-template path (tr_template_prepare + tr_verify_step_template) against the
oracle: one prepared template serves steps with different prefix lengths; what the step
returns must match the oracle exactly as the ordinary step does (and, beyond the bar, be
bit-identical to the ordinary step, since only the bookkeeping launches differ)."""
import ctypes

import numpy as np
import pytest
import torch

from gpu_util import (DEV, Batch, device_weights, fill_pool, make_template, nan_pool, oracle_cache,
                      read_pool, rel_err, run_step)
from oracle import tr_oracle as O
from paper_2406_17404_amd import binding as b
from paper_2406_17404_amd import inputs as I

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-5, "bf16": 1e-2}


def prefix_normal(shape, seed, s, L):
    return [I.gen_prefix_kv(shape, seed, l, s, L) for l in range(shape.n_layers)]


def check_against_oracle(shape, w, res, batch, trees, toks, Ls, pkvs, tol, skip=()):
    H, dh = shape.kv_heads, shape.head_dim
    for s in range(batch.B):
        if s in skip:
            continue
        L, n, r = Ls[s], len(trees[s]), batch.rows(s)
        kv = oracle_cache(shape, pkvs[s], L, n)
        want = O.decoder_tree_forward(shape, w, kv, toks[s], trees[s], L)
        assert rel_err(res["logits"][r], want) <= tol, s
        am = O.greedy_argmax(res["logits"][r])
        assert np.array_equal(res["argmax"][r], am)
        a, best, path, bonus = O.accept_path(am, toks[s], trees[s])
        assert (res["status"][s], res["accept_len"][s], res["best"][s], res["bonus"][s]) == (0, a, best, bonus)
        assert list(res["path"][s, :a + 1]) == path and (res["path"][s, a + 1:] == -1).all()
        new_len = O.kv_compact(kv, path, a, L)
        assert res["new_len"][s] == new_len
        for l in range(shape.n_layers):
            Kg, Vg = read_pool(res["k_pool"], res["v_pool"], l, batch, s, new_len, dh)
            assert rel_err(Kg, kv[l][0][:, :new_len]) <= tol and rel_err(Vg, kv[l][1][:, :new_len]) <= tol


def pools_for(shape, batch, Ls, pkvs):
    H, dh = shape.kv_heads, shape.head_dim
    kp = nan_pool(shape.n_layers, H, batch.s_pool, dh, shape.dtype)
    vp = nan_pool(shape.n_layers, H, batch.s_pool, dh, shape.dtype)
    for s in range(batch.B):
        if Ls[s]:
            for l in range(shape.n_layers):
                fill_pool(kp, vp, l, batch, s, *pkvs[s][l])
    return kp, vp


@pytest.mark.parametrize("dtype,shape_args", [("bf16", (2, 512, 4, 128, 1408, 1024)),
                                              ("f32", (2, 256, 4, 64, 1024, 2048)),
                                              ("bf16", (2, 512, 8, 64, 1408, 1024, 2))])
def test_one_template_serves_steps_with_growing_prefixes(dtype, shape_args):
    """Three sequences with different trees (a 128-node one among them); the template is
    prepared once and used for two steps whose prefixes differ, as in a decoding loop."""
    kvh = shape_args[6] if len(shape_args) > 6 else 0
    shape = I.ModelShape(*shape_args[:6], dtype, n_kv_heads=kvh)
    w = I.gen_weights(shape, 300)
    rng = np.random.default_rng(31)
    trees = [I.tree_c1(64, rng), I.tree_random(128 if dtype == "bf16" else 40, rng), I.tree_c0()]
    toks = [I.gen_tokens(shape.vocab, len(t), 300, "tree", s) for s, t in enumerate(trees)]
    desc, dw = device_weights(shape, w)
    max_pos = 640
    tmpl = None
    for step, Ls in enumerate(([70, 0, 333], [75, 9, 500])):
        pkvs = [prefix_normal(shape, 300 + step, s, L) if L else None for s, L in enumerate(Ls)]
        batch = Batch(trees, Ls, toks)
        if tmpl is None:
            tmpl = make_template(desc, batch, max_pos)
        kp, vp = pools_for(shape, batch, Ls, pkvs)
        res = run_step(shape, desc, dw, batch, kp, vp, tmpl=tmpl, max_pos=max_pos)
        check_against_oracle(shape, w, res, batch, trees, toks, Ls, pkvs, TOL[dtype])
        plain = run_step(shape, desc, dw, batch, kp, vp)
        for k in ("logits", "argmax", "accept_len", "best", "bonus", "new_len", "status", "path"):
            assert np.array_equal(res[k], plain[k]), k
        assert np.array_equal(res["k_pool"], plain["k_pool"], equal_nan=True)
        assert np.array_equal(res["v_pool"], plain["v_pool"], equal_nan=True)


def test_malformed_tree_in_the_template_and_bad_slot_ranges():
    shape = I.ModelShape(2, 512, 4, 128, 1408, 1024, "bf16")
    w = I.gen_weights(shape, 301)
    good = I.tree_c0()
    bad = good.copy()
    bad[7] = 9                       # parent with a larger index
    trees = [good, bad, good, good]
    toks = [I.gen_tokens(shape.vocab, 15, 301, "tree", s) for s in range(4)]
    Ls = [40, 10, 0, 120]
    pkvs = [prefix_normal(shape, 301, s, L) if L else None for s, L in enumerate(Ls)]
    desc, dw = device_weights(shape, w)
    batch = Batch(trees, Ls, toks)
    max_pos = 128                    # sequence 3 needs 135 positions: refused for that sequence
    tmpl = make_template(desc, batch, max_pos)
    kp, vp = pools_for(shape, batch, Ls, pkvs)
    res = run_step(shape, desc, dw, batch, kp, vp, tmpl=tmpl, max_pos=max_pos)
    assert list(res["status"]) == [0, 1, 0, 1]
    for s in (1, 3):
        assert res["accept_len"][s] == -1 and res["new_len"][s] == Ls[s] and (res["path"][s] == -1).all()
        # nothing of a marked sequence's slot range was written
        for l in range(shape.n_layers):
            o, n = int(batch.kv_off_h[s]) + Ls[s], 15
            Kg, Vg = read_pool(res["k_pool"], res["v_pool"], l, batch, s, Ls[s] + n, 128)
            assert np.isnan(Kg[:, Ls[s]:]).all() and np.isnan(Vg[:, Ls[s]:]).all()
    check_against_oracle(shape, w, res, batch, trees, toks, Ls, pkvs, 1e-2, skip=(1, 3))
    # a template made for other row ranges is not used: every sequence is marked
    tmpl2 = make_template(desc, Batch(trees, Ls, toks), 256)
    b4 = Batch([good, good, good[:14], np.concatenate([good, [0]]).astype(np.int32)], Ls,
               [t[:n] if n <= 15 else np.concatenate([t, [1]]).astype(np.int32)
                for t, n in zip(toks, (15, 15, 14, 16))])
    assert b4.T == batch.T
    kp4, vp4 = pools_for(shape, b4, Ls, pkvs)
    res4 = run_step(shape, desc, dw, b4, kp4, vp4, tmpl=tmpl2, max_pos=256)
    assert list(res4["status"]) == [0, 1, 1, 1]      # sequence 1: malformed in the template; 2, 3: other ranges


def test_template_host_side_errors():
    shape = I.ModelShape(2, 512, 4, 128, 1408, 1024, "bf16")
    desc = b.make_desc(shape)
    n = ctypes.c_size_t(0)
    l = b.lib()
    assert l.tr_template_bytes(None, 1, 15, 256, ctypes.byref(n)) == -1
    assert l.tr_template_bytes(ctypes.byref(desc), 1, 200, 256, ctypes.byref(n)) == -4
    assert l.tr_template_bytes(ctypes.byref(desc), 1, 15, 0, ctypes.byref(n)) == -2
    assert l.tr_template_bytes(ctypes.byref(desc), 1, 15, 256, ctypes.byref(n)) == 0 and n.value > 256 * 64 * 8
    t = torch.zeros(64, dtype=torch.int32, device=DEV)
    with pytest.raises(b.TrjError) as e:        # buffer too small
        b.tr_template_prepare(desc, t, t, 1, 15, 256, t)
    assert e.value.status == -5
