// Host build of the attention kernels' visibility predicate for
// tests/test_tree_visibility_cpu.py: evaluates it for a block of keys and all rows of a tree.
#include "../paper_2406_17404_amd/csrc/tree_vis.h"

extern "C" void trj_test_visible(int L, int key0, int n_keys, const uint64_t* anc, int n_rows,
                                 unsigned char* out) {
  for (int i = 0; i < n_rows; ++i)
    for (int k = 0; k < n_keys; ++k)
      out[(long)i * n_keys + k] = trj::tree_key_visible(key0 + k, L, anc[2 * i], anc[2 * i + 1]) ? 1 : 0;
}
