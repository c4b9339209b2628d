"""A plain causal decoder written with torch CPU library routines in fp64, used ONLY as
a pin for the oracle.  It knows nothing about trees, masks or acceptance: it runs an
ordinary causal forward over a token string (Eq. 1's P(y_m | y_<m, x)) and greedy
autoregressive decoding.  It shares no code with ``oracle/`` or with the HIP path:
RMSNorm, SiLU and causal attention are torch's own routines, the rotation is done with
complex multiplication."""
import torch
import torch.nn.functional as F

T64 = torch.float64


def _t(a):
    return torch.as_tensor(a, dtype=T64)


def _rotate(u, pos, theta):
    # u [n, H, dh]; pair (j, j+dh/2) is one complex number, multiplied by e^{i pos w_j}
    dh = u.shape[-1]
    half = dh // 2
    w = torch.exp(-torch.arange(half, dtype=T64) * 2.0 / dh * torch.log(_t(theta)))
    z = torch.complex(u[..., :half], u[..., half:])
    rot = torch.polar(torch.ones(len(pos), half, dtype=T64), pos.to(T64)[:, None] * w[None, :])
    z = z * rot[:, None, :]
    return torch.cat([z.real, z.imag], dim=-1)


def causal_forward(shape, weights, tokens):
    """Returns (logits[n, V], kv) where kv[l] = (K, V) as [H, n, dh] (K rotated), for an
    ordinary causal forward over `tokens` at positions 0..n-1."""
    tokens = torch.as_tensor(tokens, dtype=torch.long)
    n = len(tokens)
    H, dh, Fd = shape.n_heads, shape.head_dim, shape.d_ffn
    Hkv = getattr(shape, "n_kv_heads", 0) or H   # grouped-query: K/V heads repeated per group
    pos = torch.arange(n)
    x = _t(weights["embed"])[tokens]
    kv = []
    for w in weights["layers"]:
        h = F.rms_norm(x, (shape.d_model,), weight=_t(w["g_attn"]), eps=shape.rms_eps)
        qkv = F.linear(h, _t(w["wqkv"]))
        q, k, v = qkv.split([H * dh, Hkv * dh, Hkv * dh], dim=-1)
        q = _rotate(q.reshape(n, H, dh), pos, shape.rope_theta).transpose(0, 1)
        k = _rotate(k.reshape(n, Hkv, dh), pos, shape.rope_theta).transpose(0, 1)
        v = v.reshape(n, Hkv, dh).transpose(0, 1)
        kv.append((k.numpy().copy(), v.numpy().copy()))
        o = F.scaled_dot_product_attention(q, k.repeat_interleave(H // Hkv, dim=0),
                                           v.repeat_interleave(H // Hkv, dim=0), is_causal=True)  # [H, n, dh]
        x = x + F.linear(o.transpose(0, 1).reshape(n, H * dh), _t(w["wo"]))
        h2 = F.rms_norm(x, (shape.d_model,), weight=_t(w["g_ffn"]), eps=shape.rms_eps)
        g, u = F.linear(h2, _t(w["w_gate_up"])).split(Fd, dim=-1)
        x = x + F.linear(F.silu(g) * u, _t(w["w_down"]))
    hf = F.rms_norm(x, (shape.d_model,), weight=_t(weights["g_final"]), eps=shape.rms_eps)
    return F.linear(hf, _t(weights["w_lm"])).numpy(), kv


def greedy_decode(shape, weights, tokens, n_new):
    """Plain autoregressive greedy decoding (Eq. 1 solved first to last)."""
    toks = [int(t) for t in tokens]
    for _ in range(n_new):
        logits, _ = causal_forward(shape, weights, toks)
        toks.append(int(logits[-1].argmax()))
    return toks[len(tokens):]
