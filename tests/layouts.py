"""The tiled data layouts of include/trjacobi.h written out in numpy (index arithmetic
only), so that tests can build and read device buffers without using the library's own
converters."""
import numpy as np


def k_index(slot, c, dh):
    slot, c = np.asarray(slot), np.asarray(c)
    return ((slot // 32 * (dh // 16) + c // 16) * 64 + (c % 16) // 8 * 32 + slot % 32) * 8 + c % 8


def v_index(slot, c, dh):
    slot, c = np.asarray(slot), np.asarray(c)
    return ((((slot // 32) * (dh // 32) + c // 32) * 2 + (slot % 32) // 16) * 64
            + ((slot % 16) // 4 % 2) * 32 + c % 32) * 8 + (slot % 16) // 8 * 4 + slot % 4


def kv_to_pool(k_plain, v_plain, s_pool, slot0=0, k_pool=None, v_pool=None):
    """plain [H, n, dh] -> pool planes [H, s_pool*dh] (flat per head)."""
    H, n, dh = k_plain.shape
    if k_pool is None:
        k_pool = np.zeros((H, s_pool * dh), k_plain.dtype)
        v_pool = np.zeros((H, s_pool * dh), v_plain.dtype)
    slot = (slot0 + np.arange(n))[:, None]
    c = np.arange(dh)[None, :]
    k_pool[:, k_index(slot, c, dh)] = k_plain
    v_pool[:, v_index(slot, c, dh)] = v_plain
    return k_pool, v_pool


def pool_to_kv(k_pool, v_pool, dh, slot0, n):
    slot = (slot0 + np.arange(n))[:, None]
    c = np.arange(dh)[None, :]
    return k_pool[:, k_index(slot, c, dh)], v_pool[:, v_index(slot, c, dh)]


def logical_rows(n_out, kind, n_heads=0, dh=0):
    """logical row held by every packed row."""
    r = np.arange(n_out)
    if kind == "plain":
        return r
    t, i = r // 32, r % 32
    if kind == "gate_up":
        return np.where(i < 16, 16 * t + i, n_out // 2 + 16 * t + (i - 16))
    if kind == "qkv":
        hd = n_heads * dh                 # q rows, then k rows and v rows of equal count
        v_start = hd + (n_out - hd) // 2
        base = r // dh * dh
        j = (r % dh) // 32
        lr = base + np.where(i < 16, 16 * j + i, dh // 2 + 16 * j + (i - 16))
        return np.where(r >= v_start, r, lr)
    raise KeyError(kind)


def pack_weight(w, kind, n_heads=0, dh=0):
    """row-major [n_out, n_in] -> flat tiled buffer."""
    n_out, n_in = w.shape
    src = w[logical_rows(n_out, kind, n_heads, dh)]
    r = np.arange(n_out)[:, None]
    k = np.arange(n_in)[None, :]
    idx = ((r // 32 * (n_in // 16) + k // 16) * 64 + (k % 16) // 8 * 32 + r % 32) * 8 + k % 8
    out = np.empty(n_out * n_in, w.dtype)
    out[idx] = src
    return out
