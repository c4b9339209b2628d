"""CPU oracle for the TR-Jacobi decoding LOOP around the verify step.  TEST
INFRASTRUCTURE ONLY (same rules as ``tr_oracle.py``: only ``tests/``, the smoke check
and the benchmark's CPU leg may import it; it imports nothing from the product).

What it computes (paper, section "TR-Jacobi Decoding"): generation starts from a token
tree whose nodes are all ahead noise (Eq. 4: a token drawn at random from the tokens
that precede it); every forward verifies all paths of the tree at once, the longest
accepted path is committed together with the greedy token that follows it, and the tree
for the next round is filled from the predictions made below the accepted node in the
same forward, remaining positions again with ahead noise (paragraph "Tree-based Jacobi
Decoding").  One extra chain below the root holds retrieved tokens: the most recent
earlier occurrence of the current suffix is looked up in the committed tokens and what
followed it is proposed (paragraph "Retrieval-Augmented Jacobi Decoding", prompt
lookup).  Whatever the drafts are, the committed tokens equal plain greedy decoding
(section "Speculative Decoding"); ``tests/`` pins ``generate`` to exactly that with a
separately written autoregressive decoder.

Readings where the paper is silent (the same list is in the design notes):
  * "the path's subsequent predictions": the new tree is laid over the old one with its
    root on the accepted node `best`; a new node whose parent lies on old node u and
    which is its parent's k-th child (index order) lies on u's k-th child, if u has one;
    a new node that lies on old node w takes the prediction made at w as its token.
    For a chain this is the Jacobi update: the drafts behind the accepted run move up.
  * nodes that lie on nothing get ahead noise: token ctx[r mod len(ctx)] with r the
    (step*128 + node + 1)-th output of the SplitMix64 generator seeded with `seed`,
    ctx = all committed tokens (prompt + output so far, new root included);
  * the retrieval path is the last R nodes of the template, a chain below the root;
    prompt lookup tries suffix lengths max_ngram..1, takes the MOST RECENT earlier
    occurrence, copies up to R following tokens; unfilled retrieval nodes keep the rule
    above;
  * generation stops after max_new tokens or after the first eos token (kept).
"""
from __future__ import annotations

import numpy as np

from . import tr_oracle as O

MASK64 = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15


def splitmix64_output(seed: int, k: int) -> int:
    """k-th output (k = 1, 2, ...) of SplitMix64 started at state `seed`: the state
    advances by the golden-ratio constant per draw, the output is the state mixed by two
    xor-shift-multiply rounds and a final xor-shift."""
    z = (seed + GOLDEN * k) & MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
    return z ^ (z >> 31)


def ahead_noise(ctx, seed: int, step: int, node: int) -> int:
    """Eq. 4: a token sampled uniformly from the tokens ahead of the position."""
    return int(ctx[splitmix64_output(seed, step * 128 + node + 1) % len(ctx)])


def prompt_lookup(ctx, max_ngram: int, r: int) -> list:
    """Tokens that followed the most recent earlier occurrence of the longest matching
    suffix of ctx (suffix lengths max_ngram down to 1), at most r of them."""
    ctx = [int(t) for t in ctx]
    n_ctx = len(ctx)
    if r <= 0:
        return []
    for n in range(min(max_ngram, n_ctx - 1), 0, -1):
        suffix = ctx[n_ctx - n:]
        for i in range(n_ctx - n - 1, -1, -1):
            if ctx[i:i + n] == suffix:
                return ctx[i + n:i + n + r]
    return []


def children_lists(parent) -> list:
    ch = [[] for _ in parent]
    for i in range(1, len(parent)):
        ch[parent[i]].append(i)
    return ch


def is_retrieval_chain(parent, r: int) -> bool:
    n = len(parent)
    if r == 0:
        return True
    if r < 0 or r > n - 1:
        return False
    first = n - r
    return parent[first] == 0 and all(parent[first + j] == first + j - 1 for j in range(1, r))


def fill_tree(parent, r, ctx, max_ngram, seed, step, argmax=None, best=None) -> np.ndarray:
    """Tokens of the tree verified in round `step`.  ctx = committed tokens, its last
    one is the root.  argmax/best: predictions and accepted node of the previous round
    (None for the first tree: every node is ahead noise)."""
    n = len(parent)
    ch = children_lists(parent)
    rank = [0] * n
    for kids in ch:
        for k, v in enumerate(kids):
            rank[v] = k
    lies_on = [-1] * n
    tok = np.zeros(n, np.int32)
    tok[0] = ctx[-1]
    if best is not None:
        lies_on[0] = best
    for v in range(1, n):
        u = lies_on[parent[v]]
        if u >= 0 and rank[v] < len(ch[u]):
            lies_on[v] = ch[u][rank[v]]
        tok[v] = argmax[lies_on[v]] if lies_on[v] >= 0 else ahead_noise(ctx, seed, step, v)
    found = prompt_lookup(ctx, max_ngram, r)
    for j, t in enumerate(found):
        tok[n - r + j] = t
    return tok


def generate(shape, weights, prompt, parent, r, max_ngram, max_new, eos, seed):
    """Greedy generation by TR-Jacobi decoding.  Returns dict(tokens, accept_hist,
    n_steps): the new tokens, the number of accepted drafts of every round, the number
    of forwards after the prompt pass."""
    prompt = [int(t) for t in prompt]
    parent = np.asarray(parent, np.int32)
    if not O.validate_tree(parent) or not is_retrieval_chain(parent, r):
        raise ValueError("bad tree template")
    if len(prompt) < 1 or max_new < 1:
        raise ValueError("bad sizes")
    n = len(parent)
    cap = len(prompt) + max_new + n
    hkv = getattr(shape, "n_kv_heads", 0) or shape.n_heads
    kv = [(np.full((hkv, cap, shape.head_dim), np.nan),
           np.full((hkv, cap, shape.head_dim), np.nan)) for _ in range(shape.n_layers)]
    # prompt pass: an ordinary causal forward is the chain-shaped tree on an empty prefix
    L = len(prompt) - 1
    if L > 0:
        chain = np.arange(-1, L - 1, dtype=np.int32)
        O.decoder_tree_forward(shape, weights, kv, prompt[:L], chain, 0)
    ctx = list(prompt)
    out, hist = [], []
    argmax = best = None
    step = 0
    done = False
    while not done:
        tok = fill_tree(parent, r, ctx, max_ngram, seed, step, argmax, best)
        res = O.tr_verify_step(shape, weights, kv, tok, parent, L)
        argmax, best = res["argmax"], res["best"]
        new = [int(tok[i]) for i in res["path"][1:]] + [int(res["bonus"])]
        hist.append(res["accept_len"])
        L = res["new_len"]
        step += 1
        for t in new:
            out.append(t)
            if len(out) >= max_new or t == eos:
                done = True
                break
        ctx = list(prompt) + out if done else ctx + new
    return dict(tokens=out, accept_hist=hist, n_steps=step)
