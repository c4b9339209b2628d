// Which keys a tree node sees (appendix "Templates for Token Tree": the sparse mask of
// the token tree next to the all-ones block of the prefix).  One predicate, used by the
// attention kernels and compiled for the host by a test that checks it exhaustively
// against the tree's definition under the undefined-behaviour sanitizer (every shift
// count must lie in 0..63 for every prefix length and key).
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define TRJ_HOST_DEVICE __host__ __device__
#else
#define TRJ_HOST_DEVICE
#endif

namespace trj {

// key slot kk of a sequence with prefix length L, seen from a node whose
// ancestor-or-self bits are (anc0: nodes 0..63, anc1: nodes 64..127): prefix slots are
// always visible, slot L + j only if bit j is set, slots past node 127 never.
TRJ_HOST_DEVICE inline bool tree_key_visible(int kk, int L, uint64_t anc0, uint64_t anc1) {
  if (kk < L) return true;
  const int j = kk - L;
  return j < 64 ? ((anc0 >> j) & 1) != 0 : (j < 128 ? ((anc1 >> (j - 64)) & 1) != 0 : false);
}

}  // namespace trj
