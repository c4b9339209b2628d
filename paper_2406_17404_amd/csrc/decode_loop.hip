// TR-Jacobi decoding loop around the verify step (paper, section "TR-Jacobi Decoding"):
// host-side integer logic (ahead noise of Eq. 4, prompt lookup for the retrieval path,
// refill of the tree from the predictions below the accepted node) and the driver that
// alternates it with the device step.  One host<->device exchange per round: the tree's
// tokens and the prefix length go in, the predictions and the accepted path come out.
#include <vector>

#include "kernels.h"
#include "loop_host.h"

namespace trj {

#define TRJ_TRY(expr)              \
  do {                             \
    int rc_ = (expr);              \
    if (rc_ != TRJ_OK) return rc_; \
  } while (0)
#define TRJ_HIP(expr)              \
  do {                             \
    hipError_t e_ = (expr);        \
    if (e_ != hipSuccess) {        \
      note_hip_error(e_);          \
      return TRJ_ERR_HIP;          \
    }                              \
  } while (0)

// device-side integer blocks of the loop
struct LoopIn {   // host -> device every round
  int32_t tok[TRJ_N_MAX];
  int32_t prefix_len;
  int32_t pad[3];
};
struct LoopOut {  // device -> host every round
  int32_t argmax[TRJ_N_MAX];
  int32_t path[TRJ_N_MAX];
  int32_t accept_len, best, bonus, new_len, status;
  int32_t pad[3];
};
// A prompt pass takes up to PREFILL_CHUNKS chain-shaped trees of TRJ_N_MAX tokens in one
// packed step: chunk c is a "sequence" with the same K/V region as the others and a prefix
// that ends where chunk c - 1 ends, so its rows see the K/V that the same layer's QKV
// launch has just written for the chunks before it.  One pass over the weights then
// serves 1024 prompt tokens instead of 128.
constexpr int PREFILL_CHUNKS = 8;
struct PrefillBlock {  // host -> device every prompt pass
  int32_t tok[PREFILL_CHUNKS * TRJ_N_MAX];
  int32_t parent[PREFILL_CHUNKS * TRJ_N_MAX];
  int32_t node_off[PREFILL_CHUNKS + 1];
  int32_t kv_off[PREFILL_CHUNKS];
  int32_t prefix_len[PREFILL_CHUNKS];
  int32_t status[PREFILL_CHUNKS];
  int32_t pad[3];
};
struct LoopConst {  // host -> device once per tree shape
  int32_t parent[TRJ_N_MAX];
  int32_t node_off[2];
  int32_t kv_off;
  int32_t pad;
};

static int round_up(int x, int m) { return (x + m - 1) / m * m; }
// slot bound handed to the step for a sequence of `slots` slots: coarse, so that the
// launch shapes (and the workspace they need) take few distinct values
static int slot_bound(int slots, int s_pool) {
  int b = round_up(slots, 256);
  return b < s_pool ? b : s_pool;
}

static size_t loop_fixed_bytes() {
  return align_up(sizeof(LoopIn), 256) + align_up(sizeof(LoopOut), 256) +
         align_up(sizeof(LoopConst), 256) + align_up(sizeof(PrefillBlock), 256);
}

}  // namespace trj

using namespace trj;

extern "C" {

int32_t tr_jacobi_generate_workspace_bytes(const trj_model_desc* desc, int32_t n_nodes,
                                           int32_t prompt_len, int32_t max_new_tokens,
                                           int32_t s_pool, size_t* h_bytes) {
  if (!h_bytes) return TRJ_ERR_NULLPTR;
  TRJ_TRY(check_model(desc));
  if (n_nodes < 1 || n_nodes > TRJ_N_MAX) return TRJ_ERR_TREE_TOO_LARGE;
  if (prompt_len < 1 || max_new_tokens < 1 || s_pool < prompt_len + max_new_tokens + n_nodes)
    return TRJ_ERR_BAD_SHAPE;
  size_t need = 0;
  const int cap = prompt_len + max_new_tokens + n_nodes;
  for (int b = 256; ; b += 256) {  // every slot bound the loop can hand to the step
    int bound = b < s_pool ? b : s_pool;
    size_t a = step_workspace_bytes(*desc, 1, n_nodes, bound);
    need = a > need ? a : need;
    const int full = PREFILL_CHUNKS * TRJ_N_MAX;  // the prompt passes: full ones and the last
    for (int t : {prompt_len - 1 >= full ? full : 0, (prompt_len - 1) % full}) {
      if (t < 1 || t > bound) continue;
      a = step_workspace_bytes(*desc, (t + TRJ_N_MAX - 1) / TRJ_N_MAX, t, bound);
      need = a > need ? a : need;
    }
    if (bound >= cap || bound >= s_pool) break;
  }
  TemplateView tv;  // the rounds verify with one prepared template over cap positions
  *h_bytes = align_up(need + loop_fixed_bytes() + template_carve(nullptr, 1, n_nodes, desc->head_dim, cap, &tv), 256);
  return TRJ_OK;
}

int32_t tr_jacobi_generate(const trj_model_desc* desc, const trj_weights* weights, void* k_pool,
                           void* v_pool, size_t kv_layer_stride, int32_t s_pool,
                           const int32_t* h_prompt, int32_t prompt_len,
                           const trj_decode_config* cfg, void* workspace, size_t ws_bytes,
                           int32_t* h_tokens, int32_t* h_n_tokens, int32_t* h_accept_hist,
                           int32_t* h_n_steps, void* stream) {
  if (!cfg || !cfg->h_parent || !h_prompt || !h_tokens || !h_n_tokens || !h_n_steps || !workspace)
    return TRJ_ERR_NULLPTR;
  TRJ_TRY(check_model(desc));
  const int N = cfg->n_nodes, R = cfg->retrieval_len, max_new = cfg->max_new_tokens;
  if (N < 1 || N > TRJ_N_MAX) return TRJ_ERR_TREE_TOO_LARGE;
  if (!template_ok(cfg->h_parent, N, R) || cfg->max_ngram < 1 || max_new < 1 || prompt_len < 1)
    return TRJ_ERR_BAD_SHAPE;
  if (s_pool < prompt_len + max_new + N || (s_pool & (TRJ_KV_BLOCK - 1))) return TRJ_ERR_BAD_SHAPE;
  for (int i = 0; i < prompt_len; ++i)
    if (h_prompt[i] < 0 || h_prompt[i] >= desc->vocab) return TRJ_ERR_BAD_SHAPE;
  TuneScope tune_scope;  // one set of launch-shape knobs for the whole generation
  size_t need;
  TRJ_TRY(tr_jacobi_generate_workspace_bytes(desc, N, prompt_len, max_new, s_pool, &need));
  if (ws_bytes < need) return TRJ_ERR_WORKSPACE_TOO_SMALL;

  hipStream_t st = (hipStream_t)stream;
  char* base = static_cast<char*>(workspace);
  LoopIn* d_in = reinterpret_cast<LoopIn*>(base);
  base += align_up(sizeof(LoopIn), 256);
  LoopOut* d_out = reinterpret_cast<LoopOut*>(base);
  base += align_up(sizeof(LoopOut), 256);
  LoopConst* d_tree = reinterpret_cast<LoopConst*>(base);
  base += align_up(sizeof(LoopConst), 256);
  PrefillBlock* d_pf = reinterpret_cast<PrefillBlock*>(base);
  base += align_up(sizeof(PrefillBlock), 256);
  // the template of the decoding rounds: the tree is the same in every round (appendix
  // "Templates for Token Tree"), so its bookkeeping and the rotary table are made once
  const int max_pos = prompt_len + max_new + N;
  TemplateView tv;
  const size_t tmpl_bytes = template_carve(base, 1, N, desc->head_dim, max_pos, &tv);
  base += tmpl_bytes;
  void* step_ws = base;
  const size_t step_ws_bytes = ws_bytes - loop_fixed_bytes() - tmpl_bytes;

  LoopIn h_in{};
  LoopOut h_out{};
  LoopConst h_c{};
  *h_n_tokens = 0;
  *h_n_steps = 0;

  // ---- prompt pass: the K/V of prompt[0 .. P-2] through chain-shaped trees (an ordinary
  // causal forward), up to PREFILL_CHUNKS x TRJ_N_MAX tokens per packed step; the last
  // prompt token becomes the root
  int L = 0;
  const int n_ctx0 = prompt_len - 1;
  std::vector<PrefillBlock> h_pf_store(1);
  PrefillBlock& h_pf = h_pf_store[0];
  while (L < n_ctx0) {
    const int left = n_ctx0 - L, full = PREFILL_CHUNKS * TRJ_N_MAX;
    const int T = left < full ? left : full;
    const int Bc = (T + TRJ_N_MAX - 1) / TRJ_N_MAX;
    for (int c = 0; c < Bc; ++c) {
      const int r0 = c * TRJ_N_MAX, n = T - r0 < TRJ_N_MAX ? T - r0 : TRJ_N_MAX;
      h_pf.node_off[c] = r0;
      h_pf.kv_off[c] = 0;
      h_pf.prefix_len[c] = L + r0;
      for (int i = 0; i < n; ++i) {
        h_pf.tok[r0 + i] = h_prompt[L + r0 + i];
        h_pf.parent[r0 + i] = i - 1;
      }
    }
    h_pf.node_off[Bc] = T;
    TRJ_HIP(hipMemcpyAsync(d_pf, &h_pf, sizeof(h_pf), hipMemcpyHostToDevice, st));
    TRJ_TRY(step_impl(desc, weights, k_pool, v_pool, kv_layer_stride, s_pool, d_pf->tok, d_pf->parent,
                      d_pf->node_off, d_pf->kv_off, d_pf->prefix_len, Bc, T,
                      slot_bound(L + T, s_pool), step_ws, step_ws_bytes, nullptr, nullptr, nullptr,
                      nullptr, nullptr, nullptr, nullptr, d_pf->status, false, st));
    // the host block is reused by the next pass
    TRJ_HIP(hipStreamSynchronize(st));
    L += T;
  }

  // ---- decoding rounds
  Template tmpl;
  tmpl.build(cfg->h_parent, N);
  for (int i = 0; i < N; ++i) h_c.parent[i] = cfg->h_parent[i];
  h_c.node_off[0] = 0;
  h_c.node_off[1] = N;
  TRJ_HIP(hipMemcpyAsync(d_tree, &h_c, sizeof(h_c), hipMemcpyHostToDevice, st));
  TRJ_TRY(launch_template_prepare(d_tree->parent, d_tree->node_off, 1, N, desc->head_dim, max_pos,
                                  desc->rope_theta, tv, st));
  TRJ_HIP(hipStreamSynchronize(st));

  std::vector<int32_t> ctx(h_prompt, h_prompt + prompt_len);
  ctx.reserve(prompt_len + max_new + N);
  int n_out = 0, step = 0;
  bool have_pred = false, done = false;
  while (!done) {
    fill_tree(cfg->h_parent, tmpl, R, ctx.data(), (int)ctx.size(), cfg->max_ngram, cfg->seed, step,
              have_pred ? h_out.argmax : nullptr, h_out.best, h_in.tok);
    h_in.prefix_len = L;
    TRJ_HIP(hipMemcpyAsync(d_in, &h_in, sizeof(h_in), hipMemcpyHostToDevice, st));
    TRJ_TRY(step_impl(desc, weights, k_pool, v_pool, kv_layer_stride, s_pool, d_in->tok,
                      d_tree->parent, d_tree->node_off, &d_tree->kv_off, &d_in->prefix_len, 1, N,
                      slot_bound(L + N, s_pool), step_ws, step_ws_bytes, nullptr, d_out->argmax,
                      &d_out->accept_len, &d_out->best, d_out->path, &d_out->bonus, &d_out->new_len,
                      &d_out->status, true, st, &tv, max_pos));
    TRJ_HIP(hipMemcpyAsync(&h_out, d_out, sizeof(h_out), hipMemcpyDeviceToHost, st));
    TRJ_HIP(hipStreamSynchronize(st));
    if (h_out.status != 0 || h_out.accept_len < 0 || h_out.accept_len >= N) return TRJ_ERR_BAD_SHAPE;
    have_pred = true;
    if (h_accept_hist) h_accept_hist[step] = h_out.accept_len;
    ++step;
    const int a = h_out.accept_len;
    for (int j = 1; j <= a + 1 && !done; ++j) {
      const int32_t t = j <= a ? h_in.tok[h_out.path[j]] : h_out.bonus;
      ctx.push_back(t);
      h_tokens[n_out++] = t;
      done = n_out >= max_new || t == cfg->eos_token;
    }
    L = h_out.new_len;
  }
  *h_n_tokens = n_out;
  *h_n_steps = step;
  return TRJ_OK;
}

}  // extern "C"
