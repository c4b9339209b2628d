// The C-ABI entry points of the decoding loop that never touch the GPU (see loop_host.h).
#include "loop_host.h"

using namespace trj;

extern "C" {

uint64_t trj_splitmix64(uint64_t seed, uint64_t k) { return splitmix64_at(seed, k); }

int32_t trj_ahead_noise(const int32_t* h_ctx, int32_t ctx_len, uint64_t seed, int32_t step,
                        int32_t node, int32_t* h_token) {
  if (!h_ctx || !h_token) return TRJ_ERR_NULLPTR;
  if (ctx_len < 1 || step < 0 || node < 0 || node >= TRJ_N_MAX) return TRJ_ERR_BAD_SHAPE;
  *h_token = noise_token(h_ctx, ctx_len, seed, step, node);
  return TRJ_OK;
}

int32_t trj_prompt_lookup(const int32_t* h_ctx, int32_t ctx_len, int32_t max_ngram, int32_t r,
                          int32_t* h_out, int32_t* h_found) {
  if (!h_ctx || !h_found || (r > 0 && !h_out)) return TRJ_ERR_NULLPTR;
  if (ctx_len < 1 || max_ngram < 1 || r < 0) return TRJ_ERR_BAD_SHAPE;
  *h_found = lookup(h_ctx, ctx_len, max_ngram, r, h_out);
  return TRJ_OK;
}

int32_t trj_fill_tree(const int32_t* h_parent, int32_t n_nodes, int32_t retrieval_len,
                      const int32_t* h_ctx, int32_t ctx_len, int32_t max_ngram, uint64_t seed,
                      int32_t step, const int32_t* h_argmax, int32_t best, int32_t* h_tok) {
  if (!h_parent || !h_ctx || !h_tok) return TRJ_ERR_NULLPTR;
  if (n_nodes < 1 || n_nodes > TRJ_N_MAX) return TRJ_ERR_TREE_TOO_LARGE;
  if (!template_ok(h_parent, n_nodes, retrieval_len) || ctx_len < 1 || max_ngram < 1 || step < 0 ||
      (h_argmax && (best < 0 || best >= n_nodes)))
    return TRJ_ERR_BAD_SHAPE;
  Template t;
  t.build(h_parent, n_nodes);
  fill_tree(h_parent, t, retrieval_len, h_ctx, ctx_len, max_ngram, seed, step, h_argmax, best, h_tok);
  return TRJ_OK;
}

}  // extern "C"
