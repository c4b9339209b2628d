"""Seeded synthetic inputs for the TR-Jacobi verify step.

This module only *draws* inputs (weights, prefix K/V, token trees, tokens) with the
shapes of the five workloads; it contains none of the method's arithmetic.  Both the
CPU oracle's tests and the HIP path's tests/bench consume what it returns, so that the
two sides see identical numbers.

Everything is host-side numpy, ``numpy.random.Generator(PCG64)``, one child stream per
tensor (``SeedSequence(seed).spawn``-style keys), so any tensor can be regenerated
alone.  For bf16 workloads the values are rounded once to bf16 (round-to-nearest-even)
here and handed out as fp32 arrays holding bf16-representable numbers.

The tree shapes stand in for the paper's template (a 63-node sparse tree plus a
retrieval path of length 5, appendix "Templates for Token Tree"; draft length 4 in the
evaluation settings); the template itself is not reproduced.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Tuple

import numpy as np

N_MAX = 128  # largest tree (rows per sequence) the library accepts


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str  # "f32" or "bf16"
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    n_kv_heads: int = 0  # grouped-query attention: K/V heads (0: as many as query heads)

    @property
    def kv_heads(self) -> int:
        return self.n_kv_heads or self.n_heads


@dataclass(frozen=True)
class Workload:
    name: str
    shape: ModelShape
    seed: int
    prefix_len: Tuple[int, ...]  # one entry per sequence
    tree_kind: str  # "c0" | "c1" | "random" | "c3"
    tree_size: int


TINY = ModelShape(2, 256, 4, 64, 1024, 2048, "f32")
LLAMA7B = ModelShape(32, 4096, 32, 128, 11008, 32000, "bf16")
CODE7B = ModelShape(32, 4096, 32, 128, 11008, 32256, "bf16")
# 8B-class shape with grouped-query attention: 32 query heads share 8 K/V heads
GQA8B = ModelShape(32, 4096, 32, 128, 14336, 128256, "bf16", 1e-5, 500000.0, 8)


def workload(name: str) -> Workload:
    """The five named workloads (C0 tiny, C1 7B, C2 attention sweep has its own
    generator below, C3 long-context code model, C4 packed 16 sequences)."""
    if name == "C0":
        return Workload("C0", TINY, 1000, (128,), "c0", 15)
    if name == "C1":
        return Workload("C1", LLAMA7B, 1001, (1024,), "c1", 64)
    if name == "C3":
        return Workload("C3", CODE7B, 1003, (4096,), "c3", 128)
    if name == "G1":  # the 7B workload's recipe on the grouped-query 8B shape
        return Workload("G1", GQA8B, 1005, (1024,), "c1", 64)
    if name == "C4":
        rng = _rng(1004, "prefix_len")
        lens = tuple(int(v) for v in rng.integers(256, 4097, size=16))
        return Workload("C4", LLAMA7B, 1004, lens, "random", 64)
    raise KeyError(name)


def shrink(w: Workload, **kw) -> Workload:
    """Same workload recipe with a smaller model shape (for tests)."""
    return replace(w, shape=replace(w.shape, **kw))


# ----------------------------------------------------------------------------- rng
def _rng(seed: int, *key) -> np.random.Generator:
    """Child generator keyed by (seed, key...) so tensors are reproducible alone."""
    words = [seed]
    for k in key:
        if isinstance(k, str):
            words.extend(k.encode())
        else:
            words.append(int(k))
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(words)))


# ----------------------------------------------------------------------------- bf16
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """fp32 values rounded to the nearest bf16 (ties to even), returned as fp32."""
    u = np.array(x, dtype=np.float32, copy=True).view(np.uint32)
    t = u >> 16
    t &= 1
    t += 0x7FFF
    u += t
    u &= np.uint32(0xFFFF0000)
    return u.view(np.float32)


def _normal(rng, shape, std, dtype):
    x = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    if dtype == "bf16":  # round in place: these arrays can be hundreds of MB
        u = x.view(np.uint32)
        t = u >> 16
        t &= 1
        t += 0x7FFF
        u += t
        u &= np.uint32(0xFFFF0000)
    return x


# ----------------------------------------------------------------------------- weights
def gen_layer_weights(s: ModelShape, seed: int, layer: int) -> Dict[str, np.ndarray]:
    """One decoder layer: every matrix i.i.d. N(0, 0.02^2), row-major [out, in];
    norm gains 1.  wqkv rows are [Wq; Wk; Wv] (Wk, Wv have kv_heads * head_dim rows),
    w_gate_up rows are [Wg; Wu]."""
    d, f = s.d_model, s.d_ffn
    hd = s.n_heads * s.head_dim
    kvd = s.kv_heads * s.head_dim
    return {
        "g_attn": np.ones(d, np.float32),
        "wqkv": _normal(_rng(seed, "wqkv", layer), (hd + 2 * kvd, d), 0.02, s.dtype),
        "wo": _normal(_rng(seed, "wo", layer), (d, hd), 0.02, s.dtype),
        "g_ffn": np.ones(d, np.float32),
        "w_gate_up": _normal(_rng(seed, "wgu", layer), (2 * f, d), 0.02, s.dtype),
        "w_down": _normal(_rng(seed, "wd", layer), (d, f), 0.02, s.dtype),
    }


def gen_global_weights(s: ModelShape, seed: int) -> Dict[str, np.ndarray]:
    return {
        "embed": _normal(_rng(seed, "embed"), (s.vocab, s.d_model), 0.02, s.dtype),
        "g_final": np.ones(s.d_model, np.float32),
        "w_lm": _normal(_rng(seed, "w_lm"), (s.vocab, s.d_model), 0.02, s.dtype),
    }


def gen_weights(s: ModelShape, seed: int) -> Dict[str, object]:
    w = gen_global_weights(s, seed)
    w["layers"] = [gen_layer_weights(s, seed, l) for l in range(s.n_layers)]
    return w


# ----------------------------------------------------------------------------- trees
def tree_chain(n: int) -> np.ndarray:
    return np.arange(-1, n - 1, dtype=np.int32)


def tree_c0() -> np.ndarray:
    """15 nodes: root + 4 Jacobi drafts as a chain (0..4), two retrieval branches of 5
    hanging off the root (5..9, 10..14)."""
    p = np.empty(15, np.int32)
    p[0] = -1
    p[1:5] = np.arange(0, 4)
    p[5] = 0
    p[6:10] = np.arange(5, 9)
    p[10] = 0
    p[11:15] = np.arange(10, 14)
    return p


def tree_random(n: int, rng: np.random.Generator) -> np.ndarray:
    """parent[0] = -1, parent[i] ~ U[0, i)."""
    p = np.empty(n, np.int32)
    p[0] = -1
    for i in range(1, n):
        p[i] = rng.integers(0, i)
    return p


def tree_c1(n: int, rng: np.random.Generator, chain: int = 8, max_depth: int = 8) -> np.ndarray:
    """Nodes 0..chain-1 form the Jacobi chain (root + chain-1 drafts); every later
    node's parent is uniform over the earlier nodes whose depth is < max_depth, so no
    node is deeper than max_depth."""
    p = np.empty(n, np.int32)
    depth = np.zeros(n, np.int64)
    p[0] = -1
    for i in range(1, n):
        if i < chain:
            p[i] = i - 1
        else:
            cand = np.nonzero(depth[:i] < max_depth)[0]
            p[i] = cand[rng.integers(0, len(cand))]
        depth[i] = depth[p[i]] + 1
    return p


def tree_c3(n: int, rng: np.random.Generator, chain: int = 16) -> np.ndarray:
    """Nodes 0..chain-1 form the Jacobi chain; retrieval branches of length U{4..12}
    hang off the root until n nodes exist (the last branch is cut short)."""
    p = np.empty(n, np.int32)
    p[0] = -1
    for i in range(1, min(chain, n)):
        p[i] = i - 1
    i = chain
    while i < n:
        blen = int(rng.integers(4, 13))
        for j in range(blen):
            if i >= n:
                break
            p[i] = 0 if j == 0 else i - 1
            i += 1
    return p


def tree_template(n: int, r: int, rng: np.random.Generator) -> np.ndarray:
    """Decoding-loop template: a sparse tree of n - r nodes (tree_c1: a Jacobi chain plus
    random branches) followed by a retrieval chain of r nodes below the root."""
    jac = n - r
    p = list(tree_c1(jac, rng, chain=min(8, jac)))
    for j in range(r):
        p.append(0 if j == 0 else len(p) - 1)
    return np.asarray(p, np.int32)


def gen_trees(w: Workload) -> List[np.ndarray]:
    out = []
    for s in range(len(w.prefix_len)):
        rng = _rng(w.seed, "tree", s)
        if w.tree_kind == "c0":
            out.append(tree_c0())
        elif w.tree_kind == "c1":
            out.append(tree_c1(w.tree_size, rng))
        elif w.tree_kind == "c3":
            out.append(tree_c3(w.tree_size, rng))
        else:
            out.append(tree_random(w.tree_size, rng))
    return out


def gen_tokens(vocab: int, n: int, seed: int, *key) -> np.ndarray:
    return _rng(seed, "tok", *key).integers(0, vocab, size=n).astype(np.int32)


# ----------------------------------------------------------------------------- K/V, Q
def gen_prefix_kv(s: ModelShape, seed: int, layer: int, seq: int, length: int):
    """Prefix K and V for one layer and sequence, drawn i.i.d. N(0,1) directly (K is
    taken to be already rotated).  Returns two [kv_heads, length, head_dim] arrays."""
    k = _normal(_rng(seed, "pk", layer, seq), (s.kv_heads, length, s.head_dim), 1.0, s.dtype)
    v = _normal(_rng(seed, "pv", layer, seq), (s.kv_heads, length, s.head_dim), 1.0, s.dtype)
    return k, v


def gen_attention_case(seed: int, n_heads: int, head_dim: int, prefix: int, n: int,
                       dtype: str = "bf16", n_kv_heads: int = 0):
    """Stand-alone tree-attention case (the sweep workload): Q for n tree nodes, K/V for
    prefix+n slots (n_kv_heads of them, default one per query head), all N(0,1); a random
    parent array."""
    parent = tree_random(n, _rng(seed, "tree"))
    hk = n_kv_heads or n_heads
    q = _normal(_rng(seed, "q"), (n, n_heads, head_dim), 1.0, dtype)
    k = _normal(_rng(seed, "k"), (hk, prefix + n, head_dim), 1.0, dtype)
    v = _normal(_rng(seed, "v"), (hk, prefix + n, head_dim), 1.0, dtype)
    return q, k, v, parent


def pool_offsets(prefix_len, tree_sizes, align: int = 64):
    """Packed batches: first pool slot of every sequence (multiple of `align`) and the
    total slot count.  Sequence s owns slots [kv_off[s], kv_off[s]+prefix_len[s]+N_s)."""
    off, cur = [], 0
    for l, n in zip(prefix_len, tree_sizes):
        off.append(cur)
        cur += -(-(l + n) // align) * align
    return np.asarray(off, np.int32), cur
