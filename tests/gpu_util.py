"""Shared plumbing of the GPU parity tests: moves seeded host inputs to the device in the
library's layouts (written out independently in tests/layouts.py), runs entry points
through the binding, and brings results back as numpy."""
import numpy as np
import torch

import layouts
from oracle import tr_oracle as O
from paper_2406_17404_amd import binding as b
from paper_2406_17404_amd import inputs as I

DEV = "cuda"


def kv_heads(shape):
    return getattr(shape, "n_kv_heads", 0) or shape.n_heads


def tdtype(name):
    return torch.bfloat16 if name == "bf16" else torch.float32


def to_dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    return t.to(dtype) if dtype is not None else t


def i32(a):
    return to_dev(np.asarray(a, np.int32))


def rel_err(got, want):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    return float(np.abs(got - want).max() / max(np.abs(want).max(), 1e-30))


def device_weights(shape, w):
    """Pack a host weight dict (inputs.gen_weights) onto the device with the library."""
    desc = b.make_desc(shape)
    dt = tdtype(shape.dtype)
    dw = b.DeviceWeights(desc)
    for lw in w["layers"]:
        dw.add_layer(to_dev(lw["g_attn"].astype(np.float32)), to_dev(lw["wqkv"].astype(np.float32), dt),
                     to_dev(lw["wo"].astype(np.float32), dt), to_dev(lw["g_ffn"].astype(np.float32)),
                     to_dev(lw["w_gate_up"].astype(np.float32), dt), to_dev(lw["w_down"].astype(np.float32), dt))
    dw.set_globals(to_dev(w["embed"].astype(np.float32), dt), to_dev(w["g_final"].astype(np.float32)),
                   to_dev(w["w_lm"].astype(np.float32), dt))
    dw.finish()
    return desc, dw


class Batch:
    """Device-side description of a packed batch of trees."""

    def __init__(self, trees, prefix_len, toks=None, align=64, extra_slots=0):
        self.trees = [np.asarray(t, np.int32) for t in trees]
        self.B = len(trees)
        self.sizes = [len(t) for t in trees]
        self.T = int(sum(self.sizes))
        self.prefix_len = [int(l) for l in prefix_len]
        off, total = I.pool_offsets(self.prefix_len, self.sizes, align)
        self.kv_off_h = off
        self.s_pool = int(total + extra_slots)
        self.node_off_h = np.concatenate([[0], np.cumsum(self.sizes)]).astype(np.int32)
        self.max_seq_slots = max(l + n for l, n in zip(self.prefix_len, self.sizes))
        self.parent = i32(np.concatenate(self.trees))
        self.node_off = i32(self.node_off_h)
        self.kv_off = i32(self.kv_off_h)
        self.prefix = i32(self.prefix_len)
        self.toks_h = None if toks is None else [np.asarray(t, np.int32) for t in toks]
        self.tok = None if toks is None else i32(np.concatenate(self.toks_h))

    def rows(self, s):
        return slice(int(self.node_off_h[s]), int(self.node_off_h[s + 1]))


def nan_pool(n_layers, H, s_pool, dh, dtype_name):
    """Pool planes filled with NaN so that any read of an unwritten slot shows."""
    return np.full((n_layers, H, s_pool * dh), np.nan, np.float32)


def fill_pool(kp, vp, layer, batch, s, k_plain, v_plain):
    """Write plain [H, n, dh] rows of sequence s at the start of its slot range."""
    dh = k_plain.shape[-1]
    layouts.kv_to_pool(k_plain.astype(np.float32), v_plain.astype(np.float32), batch.s_pool,
                       int(batch.kv_off_h[s]), kp[layer], vp[layer])


def read_pool(kp, vp, layer, batch, s, n, dh):
    return layouts.pool_to_kv(kp[layer], vp[layer], dh, int(batch.kv_off_h[s]), n)


def make_template(desc, batch, max_pos):
    """A prepared tree template (device buffer) for the batch's trees."""
    tmpl = torch.empty(b.tr_template_bytes(desc, batch.B, batch.T, max_pos), dtype=torch.uint8, device=DEV)
    b.tr_template_prepare(desc, batch.parent, batch.node_off, batch.B, batch.T, max_pos, tmpl)
    return tmpl


def run_step(shape, desc, dw, batch, kp_h, vp_h, want_logits=True, tmpl=None, max_pos=0):
    """tr_verify_step (or, with a prepared template, tr_verify_step_template) through the
    binding.  kp_h / vp_h: host pools [layers, H, s_pool*dh] fp32 (bf16-representable for
    bf16 models).  Returns a dict of numpy results plus the pools after the step."""
    dt = tdtype(shape.dtype)
    kp, vp = to_dev(kp_h, dt), to_dev(vp_h, dt)
    stride = kv_heads(shape) * batch.s_pool * shape.head_dim
    ws = torch.empty(b.trj_workspace_bytes(desc, batch.T, batch.B, batch.max_seq_slots),
                     dtype=torch.uint8, device=DEV)
    B, T = batch.B, batch.T
    logits = torch.empty(T, shape.vocab, dtype=torch.float32, device=DEV) if want_logits else None
    out = {k: torch.full((n,), -7, dtype=torch.int32, device=DEV)
           for k, n in dict(argmax=T, accept_len=B, best=B, bonus=B, new_len=B, status=B).items()}
    path = torch.full((B, b.N_MAX), -7, dtype=torch.int32, device=DEV)
    head = (desc, dw.struct, kp, vp, stride, batch.s_pool, batch.tok, batch.parent, batch.node_off,
            batch.kv_off, batch.prefix, B, T, batch.max_seq_slots)
    tail = (ws, logits, out["argmax"], out["accept_len"], out["best"], path, out["bonus"],
            out["new_len"], out["status"])
    if tmpl is None:
        b.tr_verify_step(*head, *tail)
    else:
        b.tr_verify_step_template(*head, tmpl, max_pos, *tail)
    torch.cuda.synchronize()
    res = {k: v.cpu().numpy() for k, v in out.items()}
    res["path"] = path.cpu().numpy()
    res["logits"] = None if logits is None else logits.cpu().numpy()
    res["k_pool"] = kp.float().cpu().numpy()
    res["v_pool"] = vp.float().cpu().numpy()
    return res


def oracle_cache(shape, prefix_kv, L, n, pad=0):
    """fp64 cache [H, L+n+pad, dh] per layer holding the given prefix."""
    kv = []
    for l in range(shape.n_layers):
        K = np.full((kv_heads(shape), L + n + pad, shape.head_dim), np.nan)
        V = np.full_like(K, np.nan)
        if L:
            K[:, :L], V[:, :L] = prefix_kv[l]
        kv.append((K, V))
    return kv
