"""Run by tests/test_host_loop_sanitized.py in a child process whose dynamic loader has the
sanitizer runtimes preloaded: loads the sanitized build of the decoding loop's host logic
(path in argv[1]) with ctypes and checks it against the oracle on random cases, the
boundary cases included (full 128-node templates, context of one token, retrieval chains
that run into the end of the context).  Any out-of-bounds access, signed overflow or
misaligned access aborts the process with the sanitizer's report."""
import ctypes as C
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))
from oracle import tr_loop as LP   # noqa: E402


libc = C.CDLL(None)
libc.malloc.restype = C.c_void_p
libc.malloc.argtypes = [C.c_size_t]
libc.free.argtypes = [C.c_void_p]
_live = []


def exact(n):
    """n int32 in a malloc block of exactly that size (the sanitizer's redzones then sit
    right behind the last element, which Python's own allocator would not guarantee)."""
    p = libc.malloc(4 * max(1, n))
    _live.append(p)
    return C.cast(p, C.POINTER(C.c_int32))


def release():
    while _live:
        libc.free(_live.pop())


def arr(values):
    values = [int(v) for v in values]
    buf = exact(len(values))
    for i, v in enumerate(values):
        buf[i] = v
    return buf, len(values)


def template(n_jac, r, rng):
    p = [-1] + [int(rng.integers(0, i)) for i in range(1, n_jac)]
    for j in range(r):
        p.append(0 if j == 0 else len(p) - 1)
    return p


def main(path):
    lib = C.CDLL(path)
    lib.trj_splitmix64.restype = C.c_uint64
    lib.trj_splitmix64.argtypes = [C.c_uint64, C.c_uint64]
    rng = np.random.default_rng(2024)
    for seed in (0, 1234567, 2**64 - 1):
        for k in (1, 2, 1000, 2**40 + 7):
            assert lib.trj_splitmix64(seed, k) == LP.splitmix64_output(seed, k)
    n_cases = 0
    for _ in range(400):
        ctx = list(rng.integers(0, 6, size=rng.integers(1, 60)))
        cbuf, nc = arr(ctx)
        # ahead noise
        seed, step, node = int(rng.integers(0, 2**63)), int(rng.integers(0, 5000)), int(rng.integers(0, 128))
        out = C.c_int32(-1)
        assert lib.trj_ahead_noise(cbuf, nc, C.c_uint64(seed), step, node, C.byref(out)) == 0
        assert out.value == LP.ahead_noise(ctx, seed, step, node)
        # prompt lookup; the output buffer holds exactly r entries, so one write too many is caught
        ng, r = int(rng.integers(1, 6)), int(rng.integers(0, 8))
        obuf = exact(r)
        found = C.c_int32(-1)
        assert lib.trj_prompt_lookup(cbuf, nc, ng, r, obuf, C.byref(found)) == 0
        assert [int(obuf[i]) for i in range(found.value)] == list(LP.prompt_lookup(ctx, ng, r))
        # tree refill on templates of every size up to the maximum
        rr = int(rng.integers(0, 6))
        n_jac = 128 - rr if rng.random() < 0.2 else int(rng.integers(1, 128 - rr))
        parent = template(n_jac, rr, rng)
        n = len(parent)
        pbuf, _ = arr(parent)
        argmax = rng.integers(0, 32000, size=n)
        abuf, _ = arr(argmax)
        best = int(rng.integers(0, n))
        tok = exact(n)
        assert lib.trj_fill_tree(pbuf, n, rr, cbuf, nc, ng, C.c_uint64(seed), step, None, 0, tok) == 0
        assert [int(tok[i]) for i in range(n)] == list(LP.fill_tree(parent, rr, ctx, ng, seed, step))
        assert lib.trj_fill_tree(pbuf, n, rr, cbuf, nc, ng, C.c_uint64(seed), step, abuf, best, tok) == 0
        assert [int(tok[i]) for i in range(n)] == list(LP.fill_tree(parent, rr, ctx, ng, seed, step, argmax, best))
        release()
        n_cases += 1
    # argument errors must come back as codes without touching memory
    pbuf, _ = arr([-1, 2, 0])
    cbuf, _ = arr([1])
    tok = exact(3)
    assert lib.trj_fill_tree(pbuf, 3, 0, cbuf, 1, 3, C.c_uint64(0), 0, None, 0, tok) == -2
    assert lib.trj_fill_tree(pbuf, 129, 0, cbuf, 1, 3, C.c_uint64(0), 0, None, 0, tok) == -4
    assert lib.trj_prompt_lookup(cbuf, 1, 0, 2, tok, C.byref(C.c_int32(0))) == -2
    maps = open("/proc/self/maps").read()
    assert "asan" in maps and os.path.basename(path) in maps
    print(f"sanitized host logic: {n_cases} random cases equal the oracle")


if __name__ == "__main__":
    main(sys.argv[1])
