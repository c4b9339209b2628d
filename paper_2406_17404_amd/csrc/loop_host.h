// Host-side integer logic of the TR-Jacobi decoding loop (paper, section "TR-Jacobi
// Decoding"): ahead noise (Eq. 4), prompt lookup for the retrieval path, refill of the tree
// from the predictions below the accepted node.  Plain C++ with no GPU dependency, so
// that it can also be built for the host alone (e.g. under AddressSanitizer).
#pragma once
#include <stdint.h>

#include "../../include/trjacobi.h"

namespace trj {

// SplitMix64: state seed + k * golden, mixed by two xor-shift-multiply rounds
inline uint64_t splitmix64_at(uint64_t seed, uint64_t k) {
  uint64_t z = seed + 0x9E3779B97F4A7C15ull * k;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

inline int32_t noise_token(const int32_t* ctx, int32_t ctx_len, uint64_t seed, int32_t step,
                                  int32_t node) {
  uint64_t r = splitmix64_at(seed, (uint64_t)step * TRJ_N_MAX + (uint64_t)node + 1);
  return ctx[r % (uint64_t)ctx_len];
}

// longest suffix (<= max_ngram tokens) of ctx that also ends earlier in ctx; the latest
// such place wins; returns how many of the tokens that followed it were copied (<= r)
inline int lookup(const int32_t* ctx, int32_t ctx_len, int32_t max_ngram, int32_t r, int32_t* out) {
  if (r <= 0) return 0;
  int n_hi = max_ngram < ctx_len - 1 ? max_ngram : ctx_len - 1;
  for (int n = n_hi; n >= 1; --n) {
    const int32_t* suffix = ctx + ctx_len - n;
    for (int end = ctx_len - 1; end >= n; --end) {  // candidate occupies [end-n, end)
      const int32_t* cand = ctx + end - n;
      int j = n - 1;
      while (j >= 0 && cand[j] == suffix[j]) --j;
      if (j < 0) {
        int m = ctx_len - end < r ? ctx_len - end : r;
        for (int i = 0; i < m; ++i) out[i] = ctx[end + i];
        return m;
      }
    }
  }
  return 0;
}

inline bool template_ok(const int32_t* parent, int n, int r) {
  if (n < 1 || n > TRJ_N_MAX || r < 0 || r > n - 1 || parent[0] != -1) return false;
  for (int i = 1; i < n; ++i)
    if (parent[i] < 0 || parent[i] >= i) return false;
  for (int j = 0; j < r; ++j)
    if (parent[n - r + j] != (j == 0 ? 0 : n - r + j - 1)) return false;
  return true;
}

// Children in index order as a CSR list; sibling rank of every node.
struct Template {
  int n;
  int32_t first[TRJ_N_MAX + 1], kids[TRJ_N_MAX], rank[TRJ_N_MAX];
  void build(const int32_t* parent, int n_nodes) {
    n = n_nodes;
    int cnt[TRJ_N_MAX] = {0};
    for (int i = 1; i < n; ++i) cnt[parent[i]]++;
    first[0] = 0;
    for (int i = 0; i < n; ++i) first[i + 1] = first[i] + cnt[i];
    int fill[TRJ_N_MAX] = {0};
    rank[0] = 0;
    for (int i = 1; i < n; ++i) {
      int p = parent[i];
      rank[i] = fill[p];
      kids[first[p] + fill[p]++] = i;
    }
  }
  int n_kids(int u) const { return first[u + 1] - first[u]; }
};

inline void fill_tree(const int32_t* parent, const Template& t, int r, const int32_t* ctx,
                      int32_t ctx_len, int max_ngram, uint64_t seed, int step,
                      const int32_t* argmax, int best, int32_t* tok) {
  const int n = t.n;
  int32_t over[TRJ_N_MAX];  // old node under each new node, -1: none
  over[0] = argmax ? best : -1;
  tok[0] = ctx[ctx_len - 1];
  for (int v = 1; v < n; ++v) {
    int u = over[parent[v]];
    over[v] = (u >= 0 && t.rank[v] < t.n_kids(u)) ? t.kids[t.first[u] + t.rank[v]] : -1;
    tok[v] = over[v] >= 0 ? argmax[over[v]] : noise_token(ctx, ctx_len, seed, step, v);
  }
  lookup(ctx, ctx_len, max_ngram, r, tok + (n - r));
}

}  // namespace trj
