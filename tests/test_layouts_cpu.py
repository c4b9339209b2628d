"""The numpy layout formulas used by the GPU tests are bijections (CPU only)."""
import numpy as np

import layouts


def test_layout_formulas_are_bijections():
    for dh in (32, 64, 128):
        slot = np.arange(96)[:, None]
        c = np.arange(dh)[None, :]
        for f in (layouts.k_index, layouts.v_index):
            idx = f(slot, c, dh).ravel()
            assert sorted(idx) == list(range(96 * dh))


def test_row_permutations_are_bijections():
    for kind, n, H, dh in (("plain", 96, 0, 0), ("gate_up", 128, 0, 0), ("qkv", 384, 2, 64),
                           ("qkv", 3 * 3 * 128, 3, 128), ("qkv", (8 + 2 * 2) * 64, 8, 64)):
        assert sorted(layouts.logical_rows(n, kind, H, dh)) == list(range(n))
