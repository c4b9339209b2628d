"""The decoding loop through the C-ABI (tr_jacobi_generate) against the oracle's loop on
the same seeded model, prompt, template and noise seed: committed tokens, accepted drafts
per round and number of rounds, and against a separately written autoregressive greedy
decoder (the loop must not change what greedy decoding produces)."""
import numpy as np
import pytest
import torch

import brute_force_lm as BF
from gpu_util import DEV, device_weights, tdtype
from oracle import tr_loop as LP
from paper_2406_17404_amd import binding as b
from paper_2406_17404_amd import inputs as I

pytestmark = pytest.mark.gpu

F32_SHAPE = I.ModelShape(2, 64, 2, 32, 128, 64, "f32")
BF16_SHAPE = I.ModelShape(2, 128, 2, 64, 256, 96, "bf16")


def make_model(shape, seed, std=0.3):
    """Weights with a wide spread (well separated logits); bf16 models get bf16 values."""
    w = I.gen_weights(shape, seed)
    rng = np.random.default_rng(seed)
    rnd = I.bf16_round if shape.dtype == "bf16" else (lambda x: x.astype(np.float32))
    for k in ("embed", "w_lm"):
        w[k] = rnd(rng.standard_normal(w[k].shape) * std)
    for lw in w["layers"]:
        for k in ("wqkv", "wo", "w_gate_up", "w_down"):
            lw[k] = rnd(rng.standard_normal(lw[k].shape) * std / np.sqrt(lw[k].shape[1] / 32))
        lw["g_attn"] = (1 + 0.1 * rng.standard_normal(shape.d_model)).astype(np.float32)
        lw["g_ffn"] = (1 + 0.1 * rng.standard_normal(shape.d_model)).astype(np.float32)
    w["g_final"] = (1 + 0.1 * rng.standard_normal(shape.d_model)).astype(np.float32)
    return w


def hip_generate(shape, desc, dw, prompt, parent, r, max_ngram, max_new, eos, seed, slack=0):
    n = len(parent)
    s_pool = (len(prompt) + max_new + n + slack + 31) // 32 * 32
    stride = shape.kv_heads * s_pool * shape.head_dim
    dt = tdtype(shape.dtype)
    kp = torch.full((shape.n_layers, stride), float("nan"), dtype=dt, device=DEV)
    vp = torch.full((shape.n_layers, stride), float("nan"), dtype=dt, device=DEV)
    ws = torch.empty(b.tr_jacobi_generate_workspace_bytes(desc, n, len(prompt), max_new, s_pool),
                     dtype=torch.uint8, device=DEV)
    return b.tr_jacobi_generate(desc, dw.struct, kp, vp, stride, s_pool, prompt, parent, r, max_ngram,
                                max_new, eos, seed, ws)


def gap_at(shape, w, context, t_a, t_b):
    """Relative logit gap between two candidate next tokens after `context`."""
    lg, _ = BF.causal_forward(shape, w, context)
    return abs(lg[-1][t_a] - lg[-1][t_b]) / np.abs(lg[-1]).max()


@pytest.mark.parametrize("seed,n,r,plen,max_new", [(0, 12, 3, 5, 24), (1, 1, 0, 1, 8), (2, 20, 0, 9, 20),
                                                    (3, 64, 5, 140, 16), (4, 128, 5, 129, 12),
                                                    (5, 9, 4, 257, 10),
                                                    # prompt passes: one packed step of 8 chunks, then 3 chunks
                                                    (6, 10, 2, 1024 + 300, 6)])
def test_fp32_loop_equals_oracle_loop_and_autoregressive_greedy(seed, n, r, plen, max_new):
    shape = F32_SHAPE
    w = make_model(shape, seed)
    rng = np.random.default_rng(70 + seed)
    prompt = [int(t) for t in rng.integers(0, shape.vocab, size=plen)]
    parent = I.tree_template(n, r, rng)
    desc, dw = device_weights(shape, w)
    toks, hist, steps = hip_generate(shape, desc, dw, prompt, parent, r, 3, max_new, -1, seed)
    want = LP.generate(shape, w, prompt, parent, r, 3, max_new, -1, seed)
    assert toks == want["tokens"]
    assert hist == want["accept_hist"] and steps == want["n_steps"]
    if plen <= 20:
        assert toks == BF.greedy_decode(shape, w, prompt, max_new)


def test_grouped_query_loop_equals_oracle_loop():
    shape = I.ModelShape(2, 64, 4, 32, 128, 64, "f32", n_kv_heads=2)
    w = make_model(shape, 6)
    rng = np.random.default_rng(76)
    prompt = [int(t) for t in rng.integers(0, shape.vocab, size=135)]
    parent = I.tree_template(20, 4, rng)
    desc, dw = device_weights(shape, w)
    toks, hist, steps = hip_generate(shape, desc, dw, prompt, parent, 4, 3, 14, -1, 6)
    want = LP.generate(shape, w, prompt, parent, 4, 3, 14, -1, 6)
    assert toks == want["tokens"] and hist == want["accept_hist"] and steps == want["n_steps"]


def test_eos_stops_generation_and_is_kept():
    shape = F32_SHAPE
    w = make_model(shape, 0)
    prompt = [3, 1, 4, 1, 5, 9, 2, 6]
    parent = I.tree_template(12, 3, np.random.default_rng(0))
    desc, dw = device_weights(shape, w)
    full, _, _ = hip_generate(shape, desc, dw, prompt, parent, 3, 3, 20, -1, 0)
    eos = full[7]
    cut = full.index(eos) + 1
    toks, hist, steps = hip_generate(shape, desc, dw, prompt, parent, 3, 3, 20, eos, 0)
    want = LP.generate(shape, w, prompt, parent, 3, 3, 20, eos, 0)
    assert toks == full[:cut] == want["tokens"] and steps == want["n_steps"]


@pytest.mark.parametrize("seed,n,r,plen,max_new", [(0, 16, 4, 6, 24), (1, 64, 5, 150, 16), (2, 33, 0, 40, 16)])
def test_bf16_loop_against_oracle_loop(seed, n, r, plen, max_new):
    """bf16 rounding can flip a near tie, after which the two runs follow different (both
    valid) continuations: equal up to the first difference, and at that point the fp64
    logits of the two candidates are within the bf16 tolerance of each other."""
    shape = BF16_SHAPE
    w = make_model(shape, 10 + seed)
    rng = np.random.default_rng(80 + seed)
    prompt = [int(t) for t in rng.integers(0, shape.vocab, size=plen)]
    parent = I.tree_template(n, r, rng)
    desc, dw = device_weights(shape, w)
    toks, hist, steps = hip_generate(shape, desc, dw, prompt, parent, r, 3, max_new, -1, seed)
    want = LP.generate(shape, w, prompt, parent, r, 3, max_new, -1, seed)["tokens"]
    assert len(toks) == max_new and len(hist) == steps
    assert sum(a + 1 for a in hist) >= max_new > sum(a + 1 for a in hist[:-1])
    diff = [i for i in range(max_new) if toks[i] != want[i]]
    print(f"[bf16 loop] first difference: {diff[0] if diff else None}; accepted per round {hist}")
    if diff:
        i = diff[0]
        assert gap_at(shape, w, prompt + want[:i], toks[i], want[i]) <= 1e-2


def test_argument_errors():
    shape = F32_SHAPE
    w = make_model(shape, 0)
    desc, dw = device_weights(shape, w)
    parent = I.tree_template(8, 2, np.random.default_rng(0))
    s_pool = 64
    stride = shape.n_heads * s_pool * shape.head_dim
    kp = torch.zeros((shape.n_layers, stride), device=DEV)
    vp = torch.zeros_like(kp)
    ws = torch.empty(b.tr_jacobi_generate_workspace_bytes(desc, 8, 4, 8, s_pool), dtype=torch.uint8, device=DEV)
    ok = lambda **kw: b.tr_jacobi_generate(desc, dw.struct, kp, vp, stride, kw.get("s_pool", s_pool),
                                           kw.get("prompt", [1, 2, 3, 4]), kw.get("parent", parent),
                                           kw.get("r", 2), 3, kw.get("max_new", 8), -1, 0, kw.get("ws", ws))
    assert len(ok()[0]) == 8
    for bad in (dict(prompt=[1, 2, 64, 4]), dict(parent=[-1, 0, 0], r=2), dict(max_new=60),
                dict(ws=ws[:4096]), dict(s_pool=48), dict(r=8)):
        with pytest.raises(b.TrjError):
            ok(**bad)


def test_long_accepted_runs_on_a_nearly_markov_model():
    """With attention and FFN contributions scaled down the next token depends almost only
    on the current one, greedy text becomes periodic, and both the retrieved tokens and
    the model's own drafts get accepted several at a time: exercises deep accepted paths
    (and their compaction) inside the loop."""
    shape = F32_SHAPE
    w = make_model(shape, 7)
    for lw in w["layers"]:
        lw["wo"] *= 0.02
        lw["w_down"] *= 0.02
    rng = np.random.default_rng(7)
    prompt = [int(t) for t in rng.integers(0, shape.vocab, size=6)]
    parent = I.tree_template(24, 6, rng)
    desc, dw = device_weights(shape, w)
    toks, hist, steps = hip_generate(shape, desc, dw, prompt, parent, 6, 3, 96, -1, 3)
    want = LP.generate(shape, w, prompt, parent, 6, 3, 96, -1, 3)
    print(f"[markov loop] accepted per round {hist}")
    assert toks == want["tokens"] and hist == want["accept_hist"]
    assert max(hist) >= 4 and steps <= 48
