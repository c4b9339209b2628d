"""tr_verify_step through the C-ABI against the oracle on the same seeded inputs.

Tolerances (relative error = max |gpu - oracle| / max |oracle| per tensor): 1e-5 in
fp32 mode, 1e-2 in bf16 mode.  Integer outputs (argmax, accepted length, path, bonus,
new length) are compared exactly, with both sides deciding from the SAME logits (the
GPU's fp32 logits are handed to the oracle's argmax/accept), because an argmax over
nearly tied logits is not stable under any rounding difference."""
import numpy as np
import pytest

import brute_force_lm as BF
from gpu_util import (Batch, device_weights, fill_pool, nan_pool, oracle_cache, read_pool, rel_err,
                      run_step)
from oracle import tr_oracle as O
from paper_2406_17404_amd import binding as b
from paper_2406_17404_amd import inputs as I

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-5, "bf16": 1e-2}


def prefix_from_prefill(shape, w, L, seed):
    """Prefix K/V produced by the model itself (plain causal prefill of L seeded tokens)."""
    toks = I.gen_tokens(shape.vocab, L, seed, "prefix")
    _, kv = BF.causal_forward(shape, w, toks)
    if shape.dtype == "bf16":
        kv = [(I.bf16_round(k.astype(np.float32)), I.bf16_round(v.astype(np.float32))) for k, v in kv]
    return toks, kv


def prefix_normal(shape, seed, s, L):
    return [I.gen_prefix_kv(shape, seed, l, s, L) for l in range(shape.n_layers)]


def run_and_check(shape, w, trees, toks, prefix_lens, prefix_kvs, tol):
    desc, dw = device_weights(shape, w)
    batch = Batch(trees, prefix_lens, toks)
    H, dh = shape.kv_heads, shape.head_dim
    kp, vp = nan_pool(shape.n_layers, H, batch.s_pool, dh, shape.dtype), nan_pool(
        shape.n_layers, H, batch.s_pool, dh, shape.dtype)
    for s in range(batch.B):
        if prefix_lens[s]:
            for l in range(shape.n_layers):
                fill_pool(kp, vp, l, batch, s, *prefix_kvs[s][l])
    res = run_step(shape, desc, dw, batch, kp, vp)
    assert (res["status"] == 0).all()
    summary = []
    for s in range(batch.B):
        L, n, r = prefix_lens[s], len(trees[s]), batch.rows(s)
        kv = oracle_cache(shape, prefix_kvs[s], L, n)
        want = O.decoder_tree_forward(shape, w, kv, toks[s], trees[s], L)
        err = rel_err(res["logits"][r], want)
        assert err <= tol, (s, err)
        # K/V written for the tree rows, before compaction is undone by reading the
        # accepted prefix only: compare the compacted cache instead
        am = O.greedy_argmax(res["logits"][r])
        assert np.array_equal(res["argmax"][r], am)
        a, best, path, bonus = O.accept_path(am, toks[s], trees[s])
        assert (res["accept_len"][s], res["best"][s], res["bonus"][s]) == (a, best, bonus)
        assert list(res["path"][s, :a + 1]) == path and (res["path"][s, a + 1:] == -1).all()
        new_len = O.kv_compact(kv, path, a, L)
        assert res["new_len"][s] == new_len
        for l in range(shape.n_layers):
            Kg, Vg = read_pool(res["k_pool"], res["v_pool"], l, batch, s, new_len, dh)
            assert rel_err(Kg, kv[l][0][:, :new_len]) <= tol
            assert rel_err(Vg, kv[l][1][:, :new_len]) <= tol
            if L:  # the prefix itself is untouched, bit for bit
                Kp, Vp = read_pool(kp, vp, l, batch, s, L, dh)
                assert np.array_equal(Kg[:, :L], Kp) and np.array_equal(Vg[:, :L], Vp)
        # how decisive the oracle's own argmax is (reported, not asserted)
        flips = int((O.greedy_argmax(want) != am).sum())
        summary.append((err, a, flips))
    return res, summary


def test_tiny_workload_fp32():
    """Workload C0: 2 layers, d 256, 4x64 heads, FFN 1024, vocab 2048, fp32; prefix of 128
    tokens produced by a causal prefill; 15-node tree."""
    wl = I.workload("C0")
    w = I.gen_weights(wl.shape, wl.seed)
    _, pkv = prefix_from_prefill(wl.shape, w, 128, wl.seed)
    tree = I.gen_trees(wl)[0]
    tok = I.gen_tokens(wl.shape.vocab, 15, wl.seed, "tree")
    res, summary = run_and_check(wl.shape, w, [tree], [tok], [128], [pkv], 1e-5)
    print("C0 fp32 logits rel err %.2e accept %d argmax flips vs oracle %d" % summary[0])


def test_tiny_workload_fp32_planted_acceptance():
    """Drafts planted equal to the greedy continuation (computed by plain autoregressive
    decoding with the brute-force model) are fully accepted; output = greedy output."""
    wl = I.workload("C0")
    shape = wl.shape
    w = I.gen_weights(shape, wl.seed)
    # widen the weight spread so that the greedy continuation is decisive in fp32
    rng = np.random.default_rng(3)
    for lw in w["layers"]:
        for k in ("wqkv", "wo", "w_gate_up", "w_down"):
            lw[k] = (lw[k] * 3).astype(np.float32)
    w["w_lm"] = (w["w_lm"] * 10).astype(np.float32)
    ptoks, pkv = prefix_from_prefill(shape, w, 24, 5)
    root = 17
    g = BF.greedy_decode(shape, w, list(ptoks) + [root], 5)
    tree = I.tree_c0()
    tok = rng.integers(0, shape.vocab, 15).astype(np.int32)
    tok[0] = root
    tok[10:14] = g[:4]            # second retrieval branch carries the greedy continuation
    tok[14] = (g[4] + 1) % shape.vocab
    res, summary = run_and_check(shape, w, [tree], [tok], [24], [pkv], 1e-5)
    assert res["accept_len"][0] == 4 and list(res["path"][0, :5]) == [0, 10, 11, 12, 13]
    assert res["bonus"][0] == g[4]
    assert summary[0][2] == 0


@pytest.mark.parametrize("n_tree,L", [(15, 128), (64, 300), (128, 77), (1, 40), (33, 0), (69, 200), (96, 31)])
def test_small_bf16_model(n_tree, L):
    """A shrunken bf16 decoder (4 layers, d 512, 4x128 heads, FFN 1408, vocab 1024) with
    the 7B workload's recipe: N(0, 0.02) weights, N(0,1) prefix K/V, c1-style tree."""
    shape = I.ModelShape(4, 512, 4, 128, 1408, 1024, "bf16")
    w = I.gen_weights(shape, 77)
    rng = np.random.default_rng(n_tree)
    tree = I.tree_c1(n_tree, rng) if n_tree >= 8 else I.tree_chain(n_tree)
    tok = I.gen_tokens(shape.vocab, n_tree, 77, "tree", n_tree)
    pkv = prefix_normal(shape, 77, 0, L) if L else None
    res, summary = run_and_check(shape, w, [tree], [tok], [L], [pkv], 1e-2)
    print("bf16 N=%d L=%d: logits rel err %.2e accept %d flips %d" % ((n_tree, L) + summary[0]))


@pytest.mark.parametrize("dtype,tol", [("f32", 1e-5), ("bf16", 1e-2)])
@pytest.mark.parametrize("n_heads,n_kv", [(4, 2), (4, 1), (8, 2)])
def test_grouped_query_model(dtype, tol, n_heads, n_kv):
    """Grouped-query attention: n_heads query heads share n_kv K/V heads (the pool holds
    n_kv planes per layer); whole step against the oracle, packed batch of two trees."""
    dh = 128 if dtype == "bf16" else 64
    shape = I.ModelShape(2, 256, n_heads, dh, 512, 512, dtype, n_kv_heads=n_kv)
    w = I.gen_weights(shape, 88)
    rng = np.random.default_rng(n_heads * 10 + n_kv)
    trees = [I.tree_c1(40, rng), I.tree_random(9, rng)]
    Ls = [150, 0]
    toks = [I.gen_tokens(shape.vocab, len(t), 88, "tree", s) for s, t in enumerate(trees)]
    pkvs = [prefix_normal(shape, 88, 0, 150), None]
    res, summary = run_and_check(shape, w, trees, toks, Ls, pkvs, tol)
    print("gqa %s %d/%d: logits rel err %.2e" % (dtype, n_heads, n_kv, max(e for e, _, _ in summary)))


def test_packed_bf16_batch_with_ragged_prefixes():
    shape = I.ModelShape(2, 512, 4, 128, 1408, 1024, "bf16")
    w = I.gen_weights(shape, 78)
    rng = np.random.default_rng(9)
    trees, toks, Ls, pkvs = [], [], [], []
    for s in range(5):
        n = int(rng.integers(1, 65))
        L = int(rng.integers(0, 400))
        trees.append(I.tree_random(n, rng))
        toks.append(I.gen_tokens(shape.vocab, n, 78, "tree", s))
        Ls.append(L)
        pkvs.append(prefix_normal(shape, 78, s, L) if L else None)
    run_and_check(shape, w, trees, toks, Ls, pkvs, 1e-2)


@pytest.mark.parametrize("seed", range(8))
def test_random_models_and_batches(seed):
    """Random small models (width, FFN width and vocabulary any multiple of 32,
    1/2/4 query heads per K/V head, 1-3 layers) on random packed batches whose sizes sit on
    and around the tile and block boundaries; every output against the oracle."""
    rng = np.random.default_rng(4200 + seed)
    dtype = ("bf16", "f32")[seed % 2]
    dh = 128 if dtype == "bf16" else 64
    n_kv = int(rng.integers(1, 3))
    H = n_kv * int(rng.choice([1, 2, 4]))
    d = 32 * int(rng.integers(4, 13))
    ffn = 32 * int(rng.integers(5, 30))
    vocab = 32 * int(rng.integers(6, 47))
    shape = I.ModelShape(int(rng.integers(1, 4)), d, H, dh, ffn, vocab, dtype, n_kv_heads=n_kv)
    w = I.gen_weights(shape, 4300 + seed)
    trees, toks, Ls, pkvs = [], [], [], []
    rows = 0
    for s in range(int(rng.integers(1, 6))):
        n = int(rng.choice([1, 31, 32, 33, 64, 65, 128])) if rng.random() < 0.5 else int(rng.integers(1, 129))
        L = int(rng.choice([0, 31, 32, 33, 64, 255])) if rng.random() < 0.5 else int(rng.integers(0, 300))
        if rows + n > 320:
            break
        rows += n
        trees.append(I.tree_random(n, rng) if rng.random() < 0.5 else I.tree_c1(n, rng) if n >= 8 else I.tree_chain(n))
        toks.append(I.gen_tokens(shape.vocab, n, 4300 + seed, "tree", s))
        Ls.append(L)
        pkvs.append(prefix_normal(shape, 4300 + seed, s, L) if L else None)
    res, summary = run_and_check(shape, w, trees, toks, Ls, pkvs, TOL[dtype])
    print("random %s d=%d ffn=%d vocab=%d heads %d/%d layers %d, %d sequences, %d rows: worst logits rel err %.2e"
          % (dtype, d, ffn, vocab, H, n_kv, shape.n_layers, len(trees), rows, max(e for e, _, _ in summary)))


def test_packed_16_sequences_of_64_nodes():
    """The packed workload's structure (16 sequences, 64-node random trees, ragged prefixes
    U[256, 4096], 1024 tree rows in one launch) on a shrunken 2-layer model."""
    shape = I.ModelShape(2, 512, 4, 128, 1408, 1024, "bf16")
    w = I.gen_weights(shape, 1004)
    wl = I.workload("C4")
    trees = I.gen_trees(wl)
    Ls = list(wl.prefix_len)
    toks = [I.gen_tokens(shape.vocab, 64, 1004, "tree", s) for s in range(16)]
    pkvs = [prefix_normal(shape, 1004, s, Ls[s]) for s in range(16)]
    res, summary = run_and_check(shape, w, trees, toks, Ls, pkvs, 1e-2)
    print("packed 16x64: worst logits rel err %.2e" % max(e for e, _, _ in summary))


def test_long_prefix_128_node_tree():
    """The code-model workload's structure (prefix 4096, 128-node tree: chain of 16 plus
    retrieval branches) on a shrunken 2-layer model."""
    shape = I.ModelShape(2, 512, 4, 128, 1408, 1024, "bf16")
    w = I.gen_weights(shape, 1003)
    tree = I.gen_trees(I.workload("C3"))[0]
    tok = I.gen_tokens(shape.vocab, 128, 1003, "tree")
    res, summary = run_and_check(shape, w, [tree], [tok], [4096], [prefix_normal(shape, 1003, 0, 4096)], 1e-2)
    print("L=4096 N=128: logits rel err %.2e" % summary[0][0])


def test_bf16_prefill_consistent_prefix_and_planted_acceptance():
    """bf16 model whose prefix K/V come from its own prefill; drafts planted from the
    brute-force greedy continuation.  Acceptance is checked against the oracle's accept on
    the GPU's logits (exact), and against the planted length where the fp64 oracle's own
    argmaxes agree with the GPU's."""
    shape = I.ModelShape(2, 512, 4, 128, 1408, 1024, "bf16")
    w = I.gen_weights(shape, 79)
    for lw in w["layers"]:
        for k in ("wqkv", "wo", "w_gate_up", "w_down"):
            lw[k] = I.bf16_round((lw[k] * 3).astype(np.float32))
    w["w_lm"] = I.bf16_round((w["w_lm"] * 10).astype(np.float32))
    ptoks, pkv = prefix_from_prefill(shape, w, 50, 79)
    root = 5
    g = BF.greedy_decode(shape, w, list(ptoks) + [root], 7)
    tok = np.array([root] + g[:7], np.int32)
    res, summary = run_and_check(shape, w, [I.tree_chain(8)], [tok], [50], [pkv], 1e-2)
    if summary[0][2] == 0:
        assert res["accept_len"][0] == 7 and res["bonus"][0] != -1


def test_malformed_sequence_inside_a_batch():
    shape = I.ModelShape(2, 512, 4, 128, 1408, 1024, "bf16")
    w = I.gen_weights(shape, 80)
    desc, dw = device_weights(shape, w)
    good = I.tree_c0()
    bad = np.array([-1, 0, 2], np.int32)
    toks = [I.gen_tokens(1024, 15, 80, 0), np.zeros(3, np.int32), I.gen_tokens(1024, 15, 80, 2)]
    batch = Batch([good, bad, good], [40, 10, 0], toks)
    kp = nan_pool(2, 4, batch.s_pool, 128, "bf16")
    vp = nan_pool(2, 4, batch.s_pool, 128, "bf16")
    pk0 = prefix_normal(shape, 80, 0, 40)
    pk1 = prefix_normal(shape, 80, 1, 10)
    for l in range(2):
        fill_pool(kp, vp, l, batch, 0, *pk0[l])
        fill_pool(kp, vp, l, batch, 1, *pk1[l])
    res = run_step(shape, desc, dw, batch, kp, vp)
    assert list(res["status"]) == [0, 1, 0]
    assert res["accept_len"][1] == -1 and res["new_len"][1] == 10 and (res["path"][1] == -1).all()
    # the bad sequence's prefix is untouched and its tree slots were never written
    off = int(batch.kv_off_h[1]) * 128
    for l in range(2):
        a, c = res["k_pool"][l][:, off:off + 32 * 128], kp[l][:, off:off + 32 * 128]
        assert np.array_equal(np.isnan(a), np.isnan(c)) and np.array_equal(a[~np.isnan(a)], c[~np.isnan(c)])
    # the good neighbours still match the oracle
    for s, pk, L in ((0, pk0, 40), (2, None, 0)):
        kv = oracle_cache(shape, pk, L, 15)
        want = O.decoder_tree_forward(shape, w, kv, toks[s], good, L)
        assert rel_err(res["logits"][batch.rows(s)], want) <= 1e-2


def test_host_side_errors():
    import ctypes
    import torch
    shape = I.ModelShape(2, 512, 4, 128, 1408, 1024, "bf16")
    w = I.gen_weights(shape, 81)
    desc, dw = device_weights(shape, w)
    t = torch.zeros(256, dtype=torch.int32, device="cuda")
    args = lambda ws, T=15, B=1, s_pool=64, mss=55: (desc, dw.struct, t, t, 4 * 64 * 128, s_pool, t, t, t, t, t, B, T,
                                                      mss, ws, None, t, t, t, t, t, t, t)
    with pytest.raises(b.TrjError) as e:
        b.tr_verify_step(*args(t[:8]))
    assert e.value.status == -5
    with pytest.raises(b.TrjError) as e:
        b.tr_verify_step(*args(t, T=200))
    assert e.value.status == -4
    with pytest.raises(b.TrjError) as e:
        b.tr_verify_step(*args(t, s_pool=60))
    assert e.value.status == -2
    with pytest.raises(b.TrjError) as e:
        b.tr_verify_step(*args(t, mss=100))
    assert e.value.status == -2
    # widths that are not whole weight tiles are refused before anything is enqueued, in
    # both modes (the output buffers keep their contents)
    marker = torch.full((256,), 77, dtype=torch.int32, device="cuda")
    for code in (b.BF16, b.F32):
        for d_model, d_ffn in ((48, 1408), (512, 1424)):
            bad = b.ModelDesc(2, d_model, 4, 128, d_ffn, 1024, 1e-5, 1e4, code)
            with pytest.raises(b.TrjError) as e:
                b.tr_verify_step(bad, dw.struct, t, t, 4 * 64 * 128, 64, t, t, t, t, t, 1, 15, 55, t, None,
                                 marker, marker, marker, marker, marker, marker, marker)
            assert e.value.status == -2
    torch.cuda.synchronize()
    assert int((marker != 77).sum().cpu()) == 0


def test_step_can_be_captured_in_a_graph_and_replayed():
    """The step only enqueues kernels on the caller's stream (its buffers are cleared by
    fill kernels, not by memset nodes), so it can be captured in a HIP graph; every replay
    must equal the eager result, with eager work and synchronisation between replays."""
    import torch
    from gpu_util import DEV, tdtype, to_dev
    shape = I.ModelShape(2, 512, 4, 128, 1408, 1024, "bf16")
    w = I.gen_weights(shape, 31)
    desc, dw = device_weights(shape, w)
    rng = np.random.default_rng(31)
    L, n = 300, 40
    tree = I.tree_random(n, rng)
    batch = Batch([tree], [L], [I.gen_tokens(shape.vocab, n, 31, "tree")])
    stride = shape.n_heads * batch.s_pool * shape.head_dim
    g0 = torch.Generator(device=DEV).manual_seed(3)
    k0 = torch.randn(2, stride, device=DEV, generator=g0).to(torch.bfloat16)
    v0 = torch.randn(2, stride, device=DEV, generator=g0).to(torch.bfloat16)
    kp, vp = k0.clone(), v0.clone()
    ws = torch.empty(b.trj_workspace_bytes(desc, n, 1, L + n), dtype=torch.uint8, device=DEV)
    logits = torch.empty(n, shape.vocab, dtype=torch.float32, device=DEV)
    o = {k: torch.zeros(c, dtype=torch.int32, device=DEV)
         for k, c in dict(argmax=n, accept_len=1, best=1, bonus=1, new_len=1, status=1).items()}
    path = torch.zeros((1, b.N_MAX), dtype=torch.int32, device=DEV)

    def step():
        b.tr_verify_step(desc, dw.struct, kp, vp, stride, batch.s_pool, batch.tok, batch.parent,
                         batch.node_off, batch.kv_off, batch.prefix, 1, n, L + n, ws, logits, o["argmax"],
                         o["accept_len"], o["best"], path, o["bonus"], o["new_len"], o["status"])

    step()
    torch.cuda.synchronize()
    ref = {k: v.clone() for k, v in o.items()}
    ref.update(logits=logits.clone(), path=path.clone(), kp=kp.clone(), vp=vp.clone())
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        kp.copy_(k0), vp.copy_(v0)
        step()
        torch.cuda.synchronize()
        kp.copy_(k0), vp.copy_(v0)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for replay in range(4):
        kp.copy_(k0), vp.copy_(v0)
        logits.fill_(float("nan"))
        for v in o.values():
            v.fill_(-9)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in o:
            assert torch.equal(o[k], ref[k]), (replay, k)
        assert torch.equal(logits, ref["logits"]) and torch.equal(path, ref["path"]), replay
        assert torch.equal(kp, ref["kp"]) and torch.equal(vp, ref["vp"]), replay
        kp.copy_(k0), vp.copy_(v0)
        step()                       # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(logits, ref["logits"])


@pytest.mark.parametrize("n_rows,many", [(64, False), (128, False), (512, True)])
def test_argmax_in_the_lm_head_epilogue_equals_argmax_of_the_logits(n_rows, many):
    """Without a logits buffer the bf16 step takes the greedy argmax (Eq. 1) inside the LM
    head's epilogue.  Its predictions must be the oracle's argmax of the logits that the
    same step writes when it is given a buffer, ties included: the LM head here has two
    identical rows in different tiles (their logits tie wherever they are the maximum,
    the lower index must win) and zero rows everywhere else (ties at exactly 0)."""
    import torch
    from dataclasses import replace
    shape = I.ModelShape(2, 512, 4, 128, 1408, 8192 if many else 2048, "bf16")
    w = I.gen_weights(shape, 90)
    v = w["w_lm"][7].copy()
    w["w_lm"] = np.zeros_like(w["w_lm"])     # every other row ties at exactly 0
    w["w_lm"][7] = w["w_lm"][8] = w["w_lm"][1234] = v   # ties inside one tile and across tiles
    rng = np.random.default_rng(90)
    per = 128 if many else n_rows
    trees = [I.tree_random(per, rng) for _ in range(n_rows // per)]
    toks = [I.gen_tokens(shape.vocab, per, 90, "tree", s) for s in range(len(trees))]
    Ls = [int(v) for v in rng.integers(0, 200, size=len(trees))]
    pkvs = [prefix_normal(shape, 90, s, L) if L else None for s, L in enumerate(Ls)]
    if many:
        plan = b.trj_dev_gemm_plan(n_rows, shape.d_model, shape.vocab, True)
        print("LM head plan:", plan)
        assert plan["many_rows"] >= 1          # the packed-batch projection kernel takes the epilogue too
    desc, dw = device_weights(shape, w)
    batch = Batch(trees, Ls, toks)
    H, dh = shape.kv_heads, shape.head_dim
    kp, vp = nan_pool(2, H, batch.s_pool, dh, "bf16"), nan_pool(2, H, batch.s_pool, dh, "bf16")
    for s in range(batch.B):
        if Ls[s]:
            for l in range(2):
                fill_pool(kp, vp, l, batch, s, *pkvs[s][l])
    with_logits = run_step(shape, desc, dw, batch, kp, vp, want_logits=True)
    fused = run_step(shape, desc, dw, batch, kp, vp, want_logits=False)
    am = O.greedy_argmax(with_logits["logits"])
    assert np.array_equal(fused["argmax"], am)
    assert set(am.tolist()) == {0, 7}        # every row is decided by a tie: the lowest index wins
    for k in ("accept_len", "best", "bonus", "new_len", "status", "path"):
        assert np.array_equal(fused[k], with_logits[k]), k
    assert np.array_equal(fused["k_pool"], with_logits["k_pool"], equal_nan=True)
