"""ctypes binding of libtrjacobi.so: the same names and arguments as include/trjacobi.h
and include/trjacobi_dev.h.

Only argument marshalling happens here: torch tensors stand for device buffers (their
``data_ptr()`` is passed), the current torch stream is passed as the HIP stream, and a
non-zero status raises :class:`TrjError`.  Nothing is computed in Python and nothing
falls back to the CPU: if the shared library is not built, importing symbols from it
raises immediately.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# TRJ_LIB_PATH: another build of the same library (A/B measurements); default: the in-tree build
LIB_PATH = os.environ.get("TRJ_LIB_PATH") or os.path.join(_HERE, "libtrjacobi.so")

N_MAX = 128
KV_BLOCK = 32
STATIC_SCRATCH_BYTES = 32 << 20
F32, BF16 = 0, 1
PACK_PLAIN, PACK_QKV, PACK_GATE_UP = 0, 1, 2
STATUS = {0: "TRJ_OK", -1: "TRJ_ERR_NULLPTR", -2: "TRJ_ERR_BAD_SHAPE", -3: "TRJ_ERR_BAD_DTYPE",
          -4: "TRJ_ERR_TREE_TOO_LARGE", -5: "TRJ_ERR_WORKSPACE_TOO_SMALL", -6: "TRJ_ERR_HIP"}


class TrjError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__(f"{fn} returned {STATUS.get(status, status)}")


class ModelDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
                ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("dtype", C.c_int32),
                ("n_kv_heads", C.c_int32)]


class LayerWeights(C.Structure):
    _fields_ = [("g_attn", C.c_void_p), ("wqkv", C.c_void_p), ("wo", C.c_void_p),
                ("g_ffn", C.c_void_p), ("w_gate_up", C.c_void_p), ("w_down", C.c_void_p)]


class DecodeConfig(C.Structure):
    _fields_ = [("n_nodes", C.c_int32), ("h_parent", C.POINTER(C.c_int32)),
                ("retrieval_len", C.c_int32), ("max_ngram", C.c_int32),
                ("max_new_tokens", C.c_int32), ("eos_token", C.c_int32), ("seed", C.c_uint64)]


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("g_final", C.c_void_p), ("w_lm", C.c_void_p),
                ("h_layers", C.POINTER(LayerWeights))]


_lib = None
_vp, _i32, _sz, _f = C.c_void_p, C.c_int32, C.c_size_t, C.c_float
_ip = C.POINTER(C.c_int32)
_SIGS = {
    "trj_version": (C.c_char_p, []),
    "trj_last_hip_error": (_i32, []),
    "trj_set_tunable": (_i32, [C.c_char_p, _i32]),
    "trj_profile_begin": (_i32, [_i32, _i32]),
    "trj_profile_begin_span": (_i32, [_i32, _i32, _i32]),
    "trj_profile_end": (_i32, [C.POINTER(C.c_float), _i32, C.POINTER(_i32)]),
    "trj_profile_event_overhead": (_i32, [_i32, C.POINTER(C.c_float), _vp]),
    "trj_copy_probe": (_i32, [_vp, _vp, _sz, _vp]),
    "trj_read_probe": (_i32, [_vp, _sz, _vp, _vp]),
    "trj_dev_device_info": (_i32, [_ip]),
    "trj_dev_gemm_plan": (_i32, [_i32, _i32, _i32, _i32, _ip]),
    "trj_workspace_bytes": (_i32, [C.POINTER(ModelDesc), _i32, _i32, _i32, C.POINTER(_sz)]),
    "trj_pack_weight": (_i32, [_vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _vp]),
    "trj_kv_pack": (_i32, [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _vp]),
    "trj_kv_unpack": (_i32, [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _i32, _vp]),
    "trj_linear": (_i32, [_vp, _vp, _i32, _i32, _i32, _i32, _i32, _vp, _sz, _vp, _vp]),
    "trj_tree_mask": (_i32, [_vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp]),
    "tree_attention": (_i32, [_vp] * 7 + [_i32] * 8 + [_f, _vp, _sz, _vp, _vp]),
    "tree_attention_workspace_bytes": (_i32, [_i32] * 6 + [C.POINTER(_sz)]),
    "tree_attention_static_scratch": (_i32, [_vp] * 7 + [_i32] * 8 + [_f, _vp, _vp]),
    "accept_path": (_i32, [_vp] * 4 + [_i32] * 3 + [_vp] * 7),
    "kv_compact": (_i32, [_vp, _vp, _sz] + [_vp] * 4 + [_i32] * 6 + [_vp, _vp]),
    "tr_verify_step": (_i32, [C.POINTER(ModelDesc), C.POINTER(Weights), _vp, _vp, _sz, _i32] +
                       [_vp] * 5 + [_i32] * 3 + [_vp, _sz] + [_vp] * 9),
    "tr_template_bytes": (_i32, [C.POINTER(ModelDesc), _i32, _i32, _i32, C.POINTER(_sz)]),
    "tr_template_prepare": (_i32, [C.POINTER(ModelDesc), _vp, _vp, _i32, _i32, _i32, _vp, _sz, _vp]),
    "tr_verify_step_template": (_i32, [C.POINTER(ModelDesc), C.POINTER(Weights), _vp, _vp, _sz, _i32] +
                                [_vp] * 5 + [_i32] * 3 + [_vp, _sz, _i32, _vp, _sz] + [_vp] * 9),
    "trj_splitmix64": (C.c_uint64, [C.c_uint64, C.c_uint64]),
    "trj_ahead_noise": (_i32, [_ip, _i32, C.c_uint64, _i32, _i32, _ip]),
    "trj_prompt_lookup": (_i32, [_ip, _i32, _i32, _i32, _ip, _ip]),
    "trj_fill_tree": (_i32, [_ip, _i32, _i32, _ip, _i32, _i32, C.c_uint64, _i32, _ip, _i32, _ip]),
    "tr_jacobi_generate_workspace_bytes": (_i32, [C.POINTER(ModelDesc), _i32, _i32, _i32, _i32,
                                                  C.POINTER(_sz)]),
    "tr_jacobi_generate": (_i32, [C.POINTER(ModelDesc), C.POINTER(Weights), _vp, _vp, _sz, _i32,
                                  _ip, _i32, C.POINTER(DecodeConfig), _vp, _sz, _ip, _ip, _ip, _ip,
                                  _vp]),
}


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with "
                              "`python -m paper_2406_17404_amd.build` (there is no CPU fallback)")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def exported_symbols() -> List[str]:
    return list(_SIGS)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _check(fn: str, status: int):
    if status != 0:
        raise TrjError(fn, status)


def dtype_code(t: torch.dtype) -> int:
    if t == torch.float32:
        return F32
    if t == torch.bfloat16:
        return BF16
    raise ValueError(f"unsupported dtype {t}")


def trj_version() -> str:
    return lib().trj_version().decode()


def trj_set_tunable(name: str, value: int) -> None:
    _check("trj_set_tunable", lib().trj_set_tunable(name.encode(), int(value)))


KERNEL_CLASSES = {"gemm_qkv": 1, "tree_attn": 2, "attn_combine": 3, "gemm_o": 4, "reduce_norm": 5,
                  "gemm_gate_up": 6, "gemm_down": 7, "gemm_lm": 8, "argmax": 9, "accept": 10,
                  "kv_compact": 11}


def trj_profile_begin(kernel_class: int, capacity: int) -> None:
    _check("trj_profile_begin", lib().trj_profile_begin(kernel_class, capacity))


def trj_profile_begin_span(first_class: int, last_class: int, capacity: int) -> None:
    _check("trj_profile_begin_span", lib().trj_profile_begin_span(first_class, last_class, capacity))


def trj_profile_event_overhead(pairs: int = 256) -> float:
    """Milliseconds between two events recorded back to back on the current stream."""
    out = C.c_float(0)
    _check("trj_profile_event_overhead", lib().trj_profile_event_overhead(pairs, C.byref(out), _stream()))
    return float(out.value)


def trj_profile_end(capacity: int) -> List[float]:
    buf = (C.c_float * capacity)()
    n = _i32(0)
    _check("trj_profile_end", lib().trj_profile_end(buf, capacity, C.byref(n)))
    return [float(buf[i]) for i in range(n.value)]


def trj_copy_probe(dst, src, nbytes: int) -> None:
    _check("trj_copy_probe", lib().trj_copy_probe(_ptr(dst), _ptr(src), nbytes, _stream()))


def trj_read_probe(src, nbytes: int, sink) -> None:
    _check("trj_read_probe", lib().trj_read_probe(_ptr(src), nbytes, _ptr(sink), _stream()))


def trj_dev_device_info() -> dict:
    out = (C.c_int32 * 6)()
    _check("trj_dev_device_info", lib().trj_dev_device_info(out))
    return dict(zip(("compute_units", "clock_khz", "memory_clock_khz", "memory_bus_bits", "l2_bytes",
                     "lds_bytes_per_workgroup"), (int(v) for v in out)))


def trj_dev_gemm_plan(T: int, n_in: int, n_out: int, fused: bool) -> dict:
    out = (C.c_int32 * 6)()
    _check("trj_dev_gemm_plan", lib().trj_dev_gemm_plan(T, n_in, n_out, int(fused), out))
    return dict(zip(("token_tiles", "row_tiles", "k_parts", "tiles_per_wave", "split_k", "many_rows"),
                    (int(v) for v in out)))


def trj_workspace_bytes(desc: ModelDesc, t_max: int, b_max: int, l_max: int) -> int:
    n = _sz(0)
    _check("trj_workspace_bytes", lib().trj_workspace_bytes(C.byref(desc), t_max, b_max, l_max, C.byref(n)))
    return int(n.value)


def trj_pack_weight(dst, src, n_out, n_in, dtype, kind, n_heads=0, head_dim=0):
    _check("trj_pack_weight", lib().trj_pack_weight(_ptr(dst), _ptr(src), n_out, n_in, dtype, kind,
                                                    n_heads, head_dim, _stream()))


def trj_kv_pack(k_pool, v_pool, k_plain, v_plain, n_heads, head_dim, s_pool, slot0, n_slots, dtype):
    _check("trj_kv_pack", lib().trj_kv_pack(_ptr(k_pool), _ptr(v_pool), _ptr(k_plain), _ptr(v_plain),
                                            n_heads, head_dim, s_pool, slot0, n_slots, dtype, _stream()))


def trj_kv_unpack(k_plain, v_plain, k_pool, v_pool, n_heads, head_dim, s_pool, slot0, n_slots, dtype):
    _check("trj_kv_unpack", lib().trj_kv_unpack(_ptr(k_plain), _ptr(v_plain), _ptr(k_pool), _ptr(v_pool),
                                                n_heads, head_dim, s_pool, slot0, n_slots, dtype, _stream()))


def trj_linear(x, w_packed, T, n_in, n_out, dtype, split_k, workspace, y):
    _check("trj_linear", lib().trj_linear(_ptr(x), _ptr(w_packed), T, n_in, n_out, dtype, split_k,
                                          _ptr(workspace), workspace.numel() * workspace.element_size(),
                                          _ptr(y), _stream()))


def trj_tree_mask(parent, node_off, B, T, depth, anc, status_dev):
    _check("trj_tree_mask", lib().trj_tree_mask(_ptr(parent), _ptr(node_off), B, T, _ptr(depth),
                                                _ptr(anc), _ptr(status_dev), _stream()))


def tree_attention(q, k_layer, v_layer, parent, node_off, kv_off, prefix_len, B, T, n_heads,
                   head_dim, s_pool, max_seq_slots, dtype, scale, workspace, out, n_kv_heads=0):
    _check("tree_attention", lib().tree_attention(
        _ptr(q), _ptr(k_layer), _ptr(v_layer), _ptr(parent), _ptr(node_off), _ptr(kv_off),
        _ptr(prefix_len), B, T, n_heads, n_kv_heads, head_dim, s_pool, max_seq_slots, dtype, scale,
        _ptr(workspace), workspace.numel() * workspace.element_size(), _ptr(out), _stream()))


def tree_attention_workspace_bytes(B, T, n_heads, head_dim, max_seq_slots, dtype) -> int:
    n = _sz(0)
    _check("tree_attention_workspace_bytes", lib().tree_attention_workspace_bytes(
        B, T, n_heads, head_dim, max_seq_slots, dtype, C.byref(n)))
    return int(n.value)


def tree_attention_static_scratch(q, k_layer, v_layer, parent, node_off, kv_off, prefix_len, B, T,
                                  n_heads, head_dim, s_pool, max_seq_slots, dtype, scale, out,
                                  n_kv_heads=0):
    _check("tree_attention_static_scratch", lib().tree_attention_static_scratch(
        _ptr(q), _ptr(k_layer), _ptr(v_layer), _ptr(parent), _ptr(node_off), _ptr(kv_off),
        _ptr(prefix_len), B, T, n_heads, n_kv_heads, head_dim, s_pool, max_seq_slots, dtype, scale,
        _ptr(out), _stream()))


def accept_path(logits, tok, parent, node_off, B, T, V, argmax_out, accept_len, best_node, path,
                bonus_tok, status_dev):
    _check("accept_path", lib().accept_path(
        _ptr(logits), _ptr(tok), _ptr(parent), _ptr(node_off), B, T, V, _ptr(argmax_out),
        _ptr(accept_len), _ptr(best_node), _ptr(path), _ptr(bonus_tok), _ptr(status_dev), _stream()))


def kv_compact(k_pool, v_pool, kv_layer_stride, path, accept_len, kv_off, prefix_len, B, n_layers,
               n_heads, head_dim, s_pool, dtype, new_len):
    _check("kv_compact", lib().kv_compact(
        _ptr(k_pool), _ptr(v_pool), kv_layer_stride, _ptr(path), _ptr(accept_len), _ptr(kv_off),
        _ptr(prefix_len), B, n_layers, n_heads, head_dim, s_pool, dtype, _ptr(new_len), _stream()))


def tr_verify_step(desc: ModelDesc, weights: Weights, k_pool, v_pool, kv_layer_stride, s_pool, tok,
                   parent, node_off, kv_off, prefix_len, B, T, max_seq_slots, workspace, logits,
                   argmax_out, accept_len, best_node, path, bonus_tok, new_len, status_dev):
    _check("tr_verify_step", lib().tr_verify_step(
        C.byref(desc), C.byref(weights), _ptr(k_pool), _ptr(v_pool), kv_layer_stride, s_pool,
        _ptr(tok), _ptr(parent), _ptr(node_off), _ptr(kv_off), _ptr(prefix_len), B, T,
        max_seq_slots, _ptr(workspace), workspace.numel() * workspace.element_size(),
        _ptr(logits), _ptr(argmax_out), _ptr(accept_len), _ptr(best_node), _ptr(path),
        _ptr(bonus_tok), _ptr(new_len), _ptr(status_dev), _stream()))


def tr_template_bytes(desc: ModelDesc, B: int, T: int, max_pos: int) -> int:
    n = _sz(0)
    _check("tr_template_bytes", lib().tr_template_bytes(C.byref(desc), B, T, max_pos, C.byref(n)))
    return int(n.value)


def tr_template_prepare(desc: ModelDesc, parent, node_off, B, T, max_pos, tmpl) -> None:
    _check("tr_template_prepare", lib().tr_template_prepare(
        C.byref(desc), _ptr(parent), _ptr(node_off), B, T, max_pos, _ptr(tmpl),
        tmpl.numel() * tmpl.element_size(), _stream()))


def tr_verify_step_template(desc: ModelDesc, weights: Weights, k_pool, v_pool, kv_layer_stride, s_pool,
                            tok, parent, node_off, kv_off, prefix_len, B, T, max_seq_slots, tmpl,
                            max_pos, workspace, logits, argmax_out, accept_len, best_node, path,
                            bonus_tok, new_len, status_dev):
    _check("tr_verify_step_template", lib().tr_verify_step_template(
        C.byref(desc), C.byref(weights), _ptr(k_pool), _ptr(v_pool), kv_layer_stride, s_pool,
        _ptr(tok), _ptr(parent), _ptr(node_off), _ptr(kv_off), _ptr(prefix_len), B, T,
        max_seq_slots, _ptr(tmpl), tmpl.numel() * tmpl.element_size(), max_pos, _ptr(workspace),
        workspace.numel() * workspace.element_size(), _ptr(logits), _ptr(argmax_out),
        _ptr(accept_len), _ptr(best_node), _ptr(path), _ptr(bonus_tok), _ptr(new_len),
        _ptr(status_dev), _stream()))


# ------------------------------------------------------------------ decoding loop
def _host_i32(values):
    values = [int(v) for v in values]
    return (C.c_int32 * max(1, len(values)))(*values), len(values)


def trj_splitmix64(seed: int, k: int) -> int:
    return int(lib().trj_splitmix64(seed, k))


def trj_ahead_noise(ctx, seed: int, step: int, node: int) -> int:
    buf, n = _host_i32(ctx)
    out = _i32(0)
    _check("trj_ahead_noise", lib().trj_ahead_noise(buf, n, seed, step, node, C.byref(out)))
    return out.value


def trj_prompt_lookup(ctx, max_ngram: int, r: int) -> List[int]:
    buf, n = _host_i32(ctx)
    out = (C.c_int32 * max(1, r))()
    found = _i32(0)
    _check("trj_prompt_lookup", lib().trj_prompt_lookup(buf, n, max_ngram, r, out, C.byref(found)))
    return [int(out[i]) for i in range(found.value)]


def trj_fill_tree(parent, retrieval_len: int, ctx, max_ngram: int, seed: int, step: int,
                  argmax=None, best: int = 0) -> List[int]:
    pbuf, n = _host_i32(parent)
    cbuf, nc = _host_i32(ctx)
    abuf = _host_i32(argmax)[0] if argmax is not None else None
    tok = (C.c_int32 * n)()
    _check("trj_fill_tree", lib().trj_fill_tree(pbuf, n, retrieval_len, cbuf, nc, max_ngram, seed,
                                                step, abuf, best, tok))
    return [int(t) for t in tok]


def tr_jacobi_generate_workspace_bytes(desc: ModelDesc, n_nodes: int, prompt_len: int,
                                       max_new_tokens: int, s_pool: int) -> int:
    out = _sz(0)
    _check("tr_jacobi_generate_workspace_bytes", lib().tr_jacobi_generate_workspace_bytes(
        C.byref(desc), n_nodes, prompt_len, max_new_tokens, s_pool, C.byref(out)))
    return out.value


def tr_jacobi_generate(desc: ModelDesc, weights: Weights, k_pool, v_pool, kv_layer_stride, s_pool,
                       prompt, parent, retrieval_len, max_ngram, max_new_tokens, eos_token, seed,
                       workspace):
    """Returns (tokens, accept_hist, n_steps) as Python lists / int."""
    pbuf, plen = _host_i32(prompt)
    tbuf, n = _host_i32(parent)
    cfg = DecodeConfig(n, tbuf, retrieval_len, max_ngram, max_new_tokens, eos_token, seed)
    toks = (C.c_int32 * max(1, max_new_tokens))()
    hist = (C.c_int32 * max(1, max_new_tokens))()
    n_tok, n_steps = _i32(0), _i32(0)
    _check("tr_jacobi_generate", lib().tr_jacobi_generate(
        C.byref(desc), C.byref(weights), _ptr(k_pool), _ptr(v_pool), kv_layer_stride, s_pool, pbuf,
        plen, C.byref(cfg), _ptr(workspace), workspace.numel() * workspace.element_size(), toks,
        C.byref(n_tok), hist, C.byref(n_steps), _stream()))
    return ([int(toks[i]) for i in range(n_tok.value)],
            [int(hist[i]) for i in range(n_steps.value)], n_steps.value)


# ------------------------------------------------------------------ marshalling helpers
def make_desc(shape) -> ModelDesc:
    """ModelDesc from any object with the ModelShape fields (dtype "f32" / "bf16")."""
    return ModelDesc(shape.n_layers, shape.d_model, shape.n_heads, shape.head_dim, shape.d_ffn,
                     shape.vocab, shape.rms_eps, shape.rope_theta, BF16 if shape.dtype == "bf16" else F32,
                     getattr(shape, "n_kv_heads", 0))


class DeviceWeights:
    """Owns the packed device copies of a model's weights and the trj_weights struct that
    points at them.  `add_layer` / `set_globals` take row-major device tensors in the
    model dtype (norm gains fp32) and pack them with trj_pack_weight."""

    def __init__(self, desc: ModelDesc):
        self.desc = desc
        self._keep: List[torch.Tensor] = []
        self._layers: List[LayerWeights] = []
        self.struct: Optional[Weights] = None
        self._embed = self._g_final = self._w_lm = None

    def _pack(self, w: torch.Tensor, kind: int) -> torch.Tensor:
        n_out, n_in = w.shape
        dst = torch.empty_like(w)
        trj_pack_weight(dst, w.contiguous(), n_out, n_in, self.desc.dtype, kind,
                        self.desc.n_heads, self.desc.head_dim)
        self._keep.append(dst)
        return dst

    def _gain(self, g: torch.Tensor) -> torch.Tensor:
        g = g.to(torch.float32).contiguous()
        self._keep.append(g)
        return g

    def add_layer(self, g_attn, wqkv, wo, g_ffn, w_gate_up, w_down) -> None:
        self._layers.append(LayerWeights(
            self._gain(g_attn).data_ptr(), self._pack(wqkv, PACK_QKV).data_ptr(),
            self._pack(wo, PACK_PLAIN).data_ptr(), self._gain(g_ffn).data_ptr(),
            self._pack(w_gate_up, PACK_GATE_UP).data_ptr(), self._pack(w_down, PACK_PLAIN).data_ptr()))

    def set_globals(self, embed, g_final, w_lm) -> None:
        self._embed = embed.contiguous()
        self._keep.append(self._embed)
        self._g_final = self._gain(g_final)
        self._w_lm = self._pack(w_lm, PACK_PLAIN)

    def finish(self) -> Weights:
        assert len(self._layers) == self.desc.n_layers and self._embed is not None
        arr = (LayerWeights * len(self._layers))(*self._layers)
        self._arr = arr
        self.struct = Weights(self._embed.data_ptr(), self._g_final.data_ptr(),
                              self._w_lm.data_ptr(), C.cast(arr, C.POINTER(LayerWeights)))
        return self.struct
