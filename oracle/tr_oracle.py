"""CPU oracle for the TR-Jacobi verify step.  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg may
import this file; the product (the HIP library and its Python binding) never does, and
this file imports nothing from the product.  It is deliberately plain and slow: numpy,
fp64 arithmetic on whatever values it is handed, one sequence at a time, no blocking,
no fusion, no reordering.  Packed batches are a Python loop over sequences.

What it computes (paper, section "TR-Jacobi Decoding", paragraph "Tree-based Jacobi
Decoding", and appendix "Templates for Token Tree"): the draft tokens are arranged in a
token tree; ONE decoder forward scores every node, each node seeing the committed
prefix and its own ancestors only (the sparse tree-attention mask); the greedy
prediction (Eq. 1, "Jacobi Decoding") at every node is compared with the draft tokens
of its children, and the root-to-node path with the longest run of matches is kept.

Because verification must not change what greedy decoding would produce (section
"Speculative Decoding"), the result has a plain definition: the logits at node i are
the next-token logits of an ordinary causal forward over ``prefix ++ tokens on the
root-to-i path``.  ``tests/`` pins this file to that definition by brute force with a
separately written causal model, and pins the pieces below to closed forms.

Readings where the paper is silent (it never fixes an architecture, positions, a KV
cache or an acceptance formula); the same list is in the design notes:
  * architecture: pre-norm decoder, RMSNorm, rotary positions, SwiGLU FFN, no biases;
  * the root is the last committed token (always kept); a node is accepted when its
    token equals the greedy prediction at its parent and its parent is accepted;
  * a node's position is prefix_len + depth (siblings share a position);
  * rotary pairing (j, j + dh/2), angle pos * theta**(-2j/dh);
  * a node attends to every prefix token, its ancestors and itself;
  * ties: argmax -> lowest token id; equally long accepted paths -> lowest node index;
  * the accepted path's K/V rows are moved to follow the prefix contiguously;
  * grouped-query attention (the paper's general-domain base model shares K/V heads
    between query heads): query head h reads K/V head h // (n_heads // n_kv_heads).
RoPE pairing/base and the RMSNorm epsilon are conventions the paper cannot pin:
"parity unpinned" for those two choices (any self-consistent choice passes the
brute-force pin); they are pinned only to the stated closed forms.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------- tree
def validate_tree(parent) -> bool:
    """A tree is well formed when node 0 is the root and every other node's parent
    has a smaller index (topological numbering)."""
    parent = np.asarray(parent)
    if parent.ndim != 1 or len(parent) == 0 or parent[0] != -1:
        return False
    return all(0 <= int(parent[i]) < i for i in range(1, len(parent)))


def tree_depth(parent) -> np.ndarray:
    """depth[root] = 0, depth[i] = depth[parent[i]] + 1."""
    n = len(parent)
    depth = np.zeros(n, np.int32)
    for i in range(1, n):
        depth[i] = depth[parent[i]] + 1
    return depth


def ancestor_mask(parent) -> np.ndarray:
    """mask[i, j] is True when node j lies on the path root -> i (j == i included):
    the sparse attention matrix of the appendix "Templates for Token Tree"."""
    n = len(parent)
    mask = np.zeros((n, n), bool)
    for i in range(n):
        j = i
        while j != -1:
            mask[i, j] = True
            j = int(parent[j])
    return mask


def ancestor_bits(parent, words: int = 2) -> np.ndarray:
    """The same mask as bit rows: bit (j % 64) of word (j // 64) of row i."""
    mask = ancestor_mask(parent)
    n = len(parent)
    bits = np.zeros((n, words), np.uint64)
    for i in range(n):
        for j in range(n):
            if mask[i, j]:
                bits[i, j // 64] |= np.uint64(1) << np.uint64(j % 64)
    return bits


def root_path(parent, i: int) -> list:
    path = []
    while i != -1:
        path.append(int(i))
        i = int(parent[i])
    return path[::-1]


# --------------------------------------------------------------------------- layers
def rmsnorm(x, g, eps):
    """x * g / sqrt(mean(x^2) + eps) over the last axis."""
    x = np.asarray(x, F64)
    return x * np.asarray(g, F64) / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)


def rope(u, pos, theta):
    """Rotary position embedding on u[n, H, dh] at integer positions pos[n]: the pair
    (u_j, u_{j+dh/2}) is rotated by the angle pos * theta**(-2j/dh)."""
    u = np.asarray(u, F64)
    dh = u.shape[-1]
    half = dh // 2
    inv_freq = F64(theta) ** (-2.0 * np.arange(half, dtype=F64) / dh)
    ang = np.asarray(pos, F64)[:, None] * inv_freq[None, :]  # [n, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = u[..., :half], u[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(z):
    z = np.asarray(z, F64)
    return z / (1.0 + np.exp(-z))


def tree_attention(q, k, v, parent, prefix_len, scale=None, p_storage=None):
    """Tree-masked attention for one sequence.

    q[N, H, dh]; k, v[Hkv, S, dh] with S >= prefix_len + N, tree node j stored at slot
    prefix_len + j; Hkv divides H and query head h reads K/V head h // (H // Hkv)
    (Hkv == H: ordinary multi-head attention).  Node i attends to slots
    0..prefix_len-1 and to prefix_len + j for every j on its root path (itself
    included).  Returns out[N, H, dh].

    p_storage (optional, see decoder_tree_forward's `storage`): applied to the
    un-normalised weights exp(s - max s) before they multiply V, while the normalising
    sum is taken over the unrounded weights.
    """
    q = np.asarray(q, F64)
    k = np.asarray(k, F64)
    v = np.asarray(v, F64)
    n, h, dh = q.shape
    group = h // k.shape[0]
    L = int(prefix_len)
    if scale is None:
        scale = 1.0 / np.sqrt(dh)
    mask = ancestor_mask(parent)
    out = np.zeros((n, h, dh), F64)
    for i in range(n):
        slots = np.concatenate([np.arange(L), L + np.nonzero(mask[i])[0]])
        for hh in range(h):
            s = (k[hh // group, slots] @ q[i, hh]) * scale
            p = np.exp(s - s.max())
            if p_storage is None:
                p /= p.sum()
                out[i, hh] = p @ v[hh // group, slots]
            else:
                out[i, hh] = (p_storage(p) @ v[hh // group, slots]) / p.sum()
    return out


def decoder_tree_forward(shape, weights, kv, tok, parent, prefix_len, collect=None, storage=None):
    """One forward pass of the decoder over the tree's token rows (one sequence).

    shape: object with n_layers, d_model, n_heads, head_dim, d_ffn, vocab, rms_eps,
    rope_theta and optionally n_kv_heads (0 or absent: n_heads).  weights: dict with
    embed[V,d], g_final[d], w_lm[V,d] and layers[l] = {g_attn, wqkv[(H+2*Hkv)*dh, d]
    (rows Wq;Wk;Wv), wo[d, H*dh], g_ffn, w_gate_up[2F, d] (rows Wg;Wu), w_down[d, F]};
    y = x @ W.T everywhere.  kv[l] = (K, V), fp64 arrays [Hkv, S, dh]; slots
    0..prefix_len-1 hold the prefix (K already rotated); this call
    writes the tree's K/V into slots prefix_len + i.  Returns logits[N, V] (fp64).
    `collect`, if a dict, receives per-layer intermediates for kernel-level tests.

    `storage` (optional) models a reduced-precision mode, about which the paper says
    nothing (it never states the inference precision): a dict name -> callable; the
    tensors such a mode keeps in 16 bits pass through the callable where one is given:
    "h" (both normalised activations), "q", "kv" (the tree's K after rotation and V, as
    cached), "p" (attention weights, see tree_attention), "attn" (attention output),
    "act" (SiLU(gate) * up).  Everything else, and everything when storage is None (the
    default: the plain definition), stays fp64.  Tests use it to tell which rounding
    point an observed deviation comes from.
    """
    st = storage or {}
    keep = lambda name, a: st[name](a) if name in st else a
    tok = np.asarray(tok)
    n = len(tok)
    L = int(prefix_len)
    H, dh, F = shape.n_heads, shape.head_dim, shape.d_ffn
    Hkv = getattr(shape, "n_kv_heads", 0) or H
    hd, kvd = H * dh, Hkv * dh
    pos = L + tree_depth(parent)
    x = np.asarray(weights["embed"], F64)[tok]  # [n, d]
    for l in range(shape.n_layers):
        w = weights["layers"][l]
        K, V = kv[l]
        h = keep("h", rmsnorm(x, w["g_attn"], shape.rms_eps))
        qkv = h @ np.asarray(w["wqkv"], F64).T
        q = keep("q", rope(qkv[:, :hd].reshape(n, H, dh), pos, shape.rope_theta))
        kk = keep("kv", rope(qkv[:, hd:hd + kvd].reshape(n, Hkv, dh), pos, shape.rope_theta))
        vv = keep("kv", qkv[:, hd + kvd:].reshape(n, Hkv, dh))
        K[:, L:L + n] = kk.transpose(1, 0, 2)
        V[:, L:L + n] = vv.transpose(1, 0, 2)
        o = keep("attn", tree_attention(q, K, V, parent, L, p_storage=st.get("p")))
        x_mid = x + o.reshape(n, hd) @ np.asarray(w["wo"], F64).T
        h2 = keep("h", rmsnorm(x_mid, w["g_ffn"], shape.rms_eps))
        gu = h2 @ np.asarray(w["w_gate_up"], F64).T
        act = keep("act", silu(gu[:, :F]) * gu[:, F:])
        x_out = x_mid + act @ np.asarray(w["w_down"], F64).T
        if collect is not None:
            collect.setdefault("layers", []).append(
                dict(x_in=x, h=h, q=q, k=kk, v=vv, attn=o, x_mid=x_mid, h2=h2, act=act,
                     x_out=x_out))
        x = x_out
    hf = rmsnorm(x, weights["g_final"], shape.rms_eps)
    if collect is not None:
        collect["h_final"] = hf
    return hf @ np.asarray(weights["w_lm"], F64).T


# --------------------------------------------------------------------------- accept
def greedy_argmax(logits) -> np.ndarray:
    """Eq. 1's arg max per row; the lowest index wins ties, NaN never wins (a row of
    NaNs gives index 0)."""
    x = np.asarray(logits)
    x = np.where(np.isnan(x), -np.inf, x)
    return np.argmax(x, axis=-1).astype(np.int32)  # numpy returns the first maximum


def accept_path(argmax, tok, parent):
    """Longest accepted path (section "TR-Jacobi Decoding": keep the path with the
    longest accept length).  ok[0] = True; ok[i] = ok[parent[i]] and tok[i] ==
    argmax[parent[i]].  best = deepest ok node, lowest index among equals.
    Returns (accept_len, best, path, bonus): accept_len = depth[best] = number of
    accepted draft tokens, path = node indices root..best, bonus = argmax[best]."""
    n = len(parent)
    depth = tree_depth(parent)
    ok = np.zeros(n, bool)
    ok[0] = True
    for i in range(1, n):
        ok[i] = ok[parent[i]] and int(tok[i]) == int(argmax[parent[i]])
    best = 0
    for i in range(n):
        if ok[i] and depth[i] > depth[best]:
            best = i
    return int(depth[best]), best, root_path(parent, best), int(argmax[best])


def kv_compact(kv, path, accept_len, prefix_len) -> int:
    """Move the accepted path's K/V rows so that they follow the prefix: for every
    layer and head, slot prefix_len + j <- slot prefix_len + path[j], j = 0..accept_len,
    in increasing j (path[j] >= j, so no unread source is overwritten).  Returns the
    new committed length prefix_len + accept_len + 1.  Later slots are don't-care."""
    L = int(prefix_len)
    for K, V in kv:
        for j in range(accept_len + 1):
            K[:, L + j] = K[:, L + path[j]]
            V[:, L + j] = V[:, L + path[j]]
    return L + accept_len + 1


def tr_verify_step(shape, weights, kv, tok, parent, prefix_len):
    """The whole verify step for one sequence: forward, greedy argmax, longest accepted
    path, compaction.  Returns dict(logits, argmax, accept_len, best, path, bonus,
    new_len); kv is updated in place."""
    if not validate_tree(parent):
        raise ValueError("malformed tree")
    logits = decoder_tree_forward(shape, weights, kv, tok, parent, prefix_len)
    am = greedy_argmax(logits)
    a, best, path, bonus = accept_path(am, tok, parent)
    new_len = kv_compact(kv, path, a, prefix_len)
    return dict(logits=logits, argmax=am, accept_len=a, best=best, path=path, bonus=bonus,
                new_len=new_len)
