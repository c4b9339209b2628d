/*
 * libtrjacobi — the verify step of TR-Jacobi decoding on one MI355X (gfx950).
 *
 * Paper: "Make Some Noise", section "TR-Jacobi Decoding" (paragraph "Tree-based
 * Jacobi Decoding") and appendix "Templates for Token Tree".  The draft tokens of a
 * decoding round are held in a token tree; one decoder forward scores every node,
 * each node attending to the committed prefix and to its own ancestors (the sparse
 * tree-attention mask); the greedy prediction (Eq. 1) at every node is compared with
 * the draft tokens of its children and the path with the longest run of matches is
 * kept.  The paper leaves the decoder architecture, the positions of tree nodes, the
 * KV cache and the exact acceptance formula open; the readings used here are stated
 * next to each entry point.
 *
 * General rules
 *  - C linkage, plain pointers and sizes.  Every function returns a trj_status.
 *    Nothing throws, nothing aborts.
 *  - Pointers are DEVICE pointers unless the name starts with h_ (host).  The caller
 *    owns every buffer; the library allocates and frees nothing.  Process-wide state: the
 *    last HIP error code, the fixed scratch array of tree_attention_static_scratch and
 *    its per-device address, and what the development header trjacobi_dev.h adds (launch
 *    knobs, an event timer).  Entry points may be called from several threads as long as
 *    their buffers do not overlap.
 *  - Every call only enqueues work on `stream` (a hipStream_t passed as void*; NULL
 *    is the default stream) and returns; no host synchronisation happens inside.
 *  - Errors the host can see (null pointers, shapes, dtype, sizes) are returned
 *    before anything is enqueued and leave all outputs untouched.  Malformed trees
 *    are only visible on the device: they set status_dev[s] = 1 for that sequence
 *    (see accept_path).
 *
 * Tree encoding (per sequence): nodes are numbered so that parent[i] < i, node 0 is
 * the root with parent[0] = -1.  The root is the last committed token; its K/V is not
 * in the cache yet and it is always kept, so a step emits accept_len + 1 tokens.  At
 * most TRJ_N_MAX nodes per sequence.  Parent indices are local to the sequence.
 *
 * Packed batches: B sequences, T tree rows in total.  node_off[B+1] gives each
 * sequence's row range, kv_off[B] its first slot in the KV pool (a multiple of
 * TRJ_KV_BLOCK), prefix_len[B] its committed length.  Sequence s owns pool slots
 * [kv_off[s], kv_off[s] + prefix_len[s] + N_s); tree node i lives at slot
 * kv_off[s] + prefix_len[s] + i.
 *
 * Data layouts (element offsets; elements are 2 bytes for TRJ_BF16, 4 for TRJ_F32)
 *  - KV pool, one layer: K and V each hold one plane per K/V head (n_kv_heads, which is
 *    n_heads unless the model uses grouped-query attention) of s_pool * head_dim
 *    elements (s_pool a multiple of TRJ_KV_BLOCK, head_dim a multiple of 32); K is
 *    stored already rotated.  Inside a plane the slots are tiled in blocks of 32 so
 *    that a wavefront's 16-byte-per-lane load is one contiguous 1 KiB read that is
 *    already an MFMA operand:
 *      K(slot, c): ((slot/32 * head_dim/16 + c/16) * 64 + (c%16)/8 * 32 + slot%32) * 8 + c%8
 *      V(slot, c): (((slot/32 * head_dim/32 + c/32) * 2 + (slot%32)/16) * 64
 *                   + ((slot%16)/4 % 2) * 32 + c%32) * 8 + (slot%16)/8 * 4 + slot%4
 *    trj_kv_pack / trj_kv_unpack convert from / to plain [head][slot][head_dim].
 *    All layers: layer l starts kv_layer_stride elements after layer l-1.
 *  - Weight matrices W[n_out][n_in] (y = x W^T, no biases) are tiled 32 rows x 16
 *    columns by trj_pack_weight:
 *      W(r, k): ((r/32 * n_in/16 + k/16) * 64 + (k%16)/8 * 32 + r%32) * 8 + k%8
 *    where r is the packed row.  TRJ_PACK_PLAIN: r = n.  TRJ_PACK_GATE_UP (rows
 *    [Wg; Wu]): tile t holds gate rows 16t..16t+15 then up rows 16t..16t+15.
 *    TRJ_PACK_QKV (rows [Wq; Wk; Wv], head-major): inside every q and k head the tile
 *    j (0..head_dim/32-1) holds dims 16j..16j+15 then head_dim/2+16j.. (the rotary
 *    partners); v rows keep their order.
 *  - q and the attention output: plain [T][n_heads][head_dim].  Logits: [T][vocab]
 *    fp32.  Norm gains: fp32 [d_model].
 */
#ifndef TRJACOBI_H
#define TRJACOBI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TRJ_N_MAX 128
#define TRJ_KV_BLOCK 32

typedef enum {
  TRJ_OK = 0,
  TRJ_ERR_NULLPTR = -1,
  TRJ_ERR_BAD_SHAPE = -2,
  TRJ_ERR_BAD_DTYPE = -3,
  TRJ_ERR_TREE_TOO_LARGE = -4,
  TRJ_ERR_WORKSPACE_TOO_SMALL = -5,
  TRJ_ERR_HIP = -6
} trj_status;

typedef enum { TRJ_F32 = 0, TRJ_BF16 = 1 } trj_dtype;
typedef enum { TRJ_PACK_PLAIN = 0, TRJ_PACK_QKV = 1, TRJ_PACK_GATE_UP = 2 } trj_pack_kind;

typedef struct {
  int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
  float rms_eps;    /* RMSNorm: x * g / sqrt(mean(x^2) + rms_eps) */
  float rope_theta; /* rotary base; pair (j, j+head_dim/2), angle pos*theta^(-2j/head_dim) */
  int32_t dtype;    /* trj_dtype of weights, KV pool and q; accumulation is fp32 */
  int32_t n_kv_heads; /* grouped-query attention: K/V heads, a divisor of n_heads; query head h
                       * reads K/V head h / (n_heads / n_kv_heads).  0 means n_heads. */
} trj_model_desc;

typedef struct {
  const float* g_attn;   /* [d_model] */
  const void* wqkv;      /* [(n_heads + 2*n_kv_heads)*head_dim][d_model], rows Wq;Wk;Wv, TRJ_PACK_QKV */
  const void* wo;        /* [d_model][n_heads*head_dim],   TRJ_PACK_PLAIN */
  const float* g_ffn;    /* [d_model] */
  const void* w_gate_up; /* [2*d_ffn][d_model],            TRJ_PACK_GATE_UP */
  const void* w_down;    /* [d_model][d_ffn],              TRJ_PACK_PLAIN */
} trj_layer_weights;

typedef struct {
  const void* embed;     /* [vocab][d_model], plain row-major, model dtype */
  const float* g_final;  /* [d_model] */
  const void* w_lm;      /* [vocab][d_model], TRJ_PACK_PLAIN */
  const trj_layer_weights* h_layers; /* HOST array of n_layers entries (device pointers inside) */
} trj_weights;

const char* trj_version(void);
/* hipError_t of the last failing HIP call seen by this library (0 if none). */
int32_t trj_last_hip_error(void);

/* Bytes of device scratch tr_verify_step / tree_attention need for a call with T = t_max
 * tree rows, B = b_max sequences and max_seq_slots = l_max.  The size is not monotonic in
 * these numbers: query every shape that will be used and take the largest.  A call whose
 * workspace is too small returns TRJ_ERR_WORKSPACE_TOO_SMALL and does nothing. */
int32_t trj_workspace_bytes(const trj_model_desc* desc, int32_t t_max, int32_t b_max,
                            int32_t l_max, size_t* h_bytes);

/* Layout helpers (see the layout section above).  src and dst must not overlap. */
int32_t trj_pack_weight(void* dst, const void* src_rowmajor, int32_t n_out, int32_t n_in,
                        int32_t dtype, int32_t kind, int32_t n_heads, int32_t head_dim,
                        void* stream);
/* plain [n_heads][n_slots][head_dim] <-> the tiled pool planes of one layer, slots
 * slot0 .. slot0+n_slots-1 of the pool.  n_heads here counts planes, i.e. K/V heads. */
int32_t trj_kv_pack(void* k_pool, void* v_pool, const void* k_plain, const void* v_plain,
                    int32_t n_heads, int32_t head_dim, int32_t s_pool, int32_t slot0,
                    int32_t n_slots, int32_t dtype, void* stream);
int32_t trj_kv_unpack(void* k_plain, void* v_plain, const void* k_pool, const void* v_pool,
                      int32_t n_heads, int32_t head_dim, int32_t s_pool, int32_t slot0,
                      int32_t n_slots, int32_t dtype, void* stream);

/* Tree bookkeeping: depth[i] = depth[parent[i]] + 1 (root 0) and the ancestor-or-self
 * bit rows of the sparse tree mask (appendix "Templates for Token Tree"): bit j%64 of
 * anc[i][j/64] is set when node j is on the path root..i.  A sequence whose tree is
 * malformed (parent[0] != -1, parent[i] outside [0, i), more than TRJ_N_MAX rows) gets
 * status_dev[s] = 1 and zeroed rows.  Outputs: depth[T], anc[T][2] (uint64),
 * status_dev[B]. */
int32_t trj_tree_mask(const int32_t* parent, const int32_t* node_off, int32_t B, int32_t T,
                      int32_t* depth, uint64_t* anc, int32_t* status_dev, void* stream);

/* Tree-masked attention for one layer (section "TR-Jacobi Decoding": every path runs
 * an ordinary Jacobi step through tree attention).  For row i of sequence s and each
 * head: softmax over {prefix slots 0..prefix_len[s]-1} U {tree slots of i's ancestors
 * and i itself} of scale * q.k, times V.  The tree's own K/V must already be in the
 * pool at slots kv_off[s] + prefix_len[s] + i.  q, out: [T][n_heads][head_dim] in
 * `dtype`.  k_layer, v_layer hold n_kv_heads planes (0: n_heads); with fewer K/V heads
 * than query heads, query head h reads plane h / (n_heads / n_kv_heads) (grouped-query
 * attention).  max_seq_slots: host upper bound of prefix_len[s] + N_s (sizes the
 * launch).  workspace: device scratch of at least trj_workspace_bytes(...) bytes. */
int32_t tree_attention(const void* q, const void* k_layer, const void* v_layer,
                       const int32_t* parent, const int32_t* node_off, const int32_t* kv_off,
                       const int32_t* prefix_len, int32_t B, int32_t T, int32_t n_heads,
                       int32_t n_kv_heads, int32_t head_dim, int32_t s_pool,
                       int32_t max_seq_slots, int32_t dtype, float scale, void* workspace,
                       size_t ws_bytes, void* out, void* stream);

/* Bytes of device scratch tree_attention alone needs at these sizes (at most what
 * trj_workspace_bytes reports for a model with these heads). */
int32_t tree_attention_workspace_bytes(int32_t B, int32_t T, int32_t n_heads, int32_t head_dim,
                                       int32_t max_seq_slots, int32_t dtype, size_t* h_bytes);

/* tree_attention for callers that cannot allocate device memory or pass a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
 * the same kernels and results, with the scratch in a fixed array of
 * TRJ_STATIC_SCRATCH_BYTES inside the library (every GPU the library runs on holds one
 * copy until the process ends).  A call for which tree_attention_workspace_bytes reports
 * more than that returns TRJ_ERR_WORKSPACE_TOO_SMALL and does nothing (the need is the
 * partial sums of sequences whose keys are split over several workgroups: 8 to 17 MiB for
 * one to four sequences with 32 heads of 128 at any length, little for larger batches;
 * more only when a development knob asks for more splits).  No
 * hipMalloc, hipFree or other allocating call is made.  All calls on one GPU share that
 * GPU's array: calls that overlap in time on one GPU (two streams, two threads) race;
 * calls on one stream are ordered and safe.  Nothing in the array needs clearing between
 * calls: every call rewrites what it reads. */
#define TRJ_STATIC_SCRATCH_BYTES (32u << 20)
int32_t tree_attention_static_scratch(const void* q, const void* k_layer, const void* v_layer,
                                      const int32_t* parent, const int32_t* node_off,
                                      const int32_t* kv_off, const int32_t* prefix_len, int32_t B,
                                      int32_t T, int32_t n_heads, int32_t n_kv_heads,
                                      int32_t head_dim, int32_t s_pool, int32_t max_seq_slots,
                                      int32_t dtype, float scale, void* out, void* stream);

/* Greedy argmax (Eq. 1) and the longest accepted path (section "TR-Jacobi Decoding").
 * If logits != NULL: argmax_out[i] = lowest index of the row maximum of logits[i][0..V)
 * (NaN never wins).  If logits == NULL, argmax_out must already hold the predictions.
 * ok[root] = 1, ok[i] = ok[parent[i]] && tok[i] == argmax_out[parent[i]]; best = the
 * deepest ok node, lowest index among equals.  Outputs per sequence: accept_len =
 * depth[best] (accepted drafts), best_node, path[s][TRJ_N_MAX] = node indices root..best
 * then -1, bonus_tok = argmax_out[best].  Malformed tree: status_dev[s] = 1,
 * accept_len[s] = -1, best_node = -1, path all -1, bonus_tok = -1. */
int32_t accept_path(const float* logits, const int32_t* tok, const int32_t* parent,
                    const int32_t* node_off, int32_t B, int32_t T, int32_t V,
                    int32_t* argmax_out, int32_t* accept_len, int32_t* best_node,
                    int32_t* path, int32_t* bonus_tok, int32_t* status_dev, void* stream);

/* In-place compaction of the accepted path (the paper has no cache; this keeps the
 * accepted rows contiguous after the prefix): for every layer and head and
 * j = 0..accept_len[s], slot kv_off+prefix_len+j <- slot kv_off+prefix_len+path[s][j]
 * for K and V; new_len[s] = prefix_len[s] + accept_len[s] + 1.  Sequences with
 * accept_len[s] < 0 are skipped (new_len = prefix_len).  Slots beyond new_len are
 * unspecified afterwards.  n_heads counts the planes of a layer, i.e. K/V heads. */
int32_t kv_compact(void* k_pool, void* v_pool, size_t kv_layer_stride, const int32_t* path,
                   const int32_t* accept_len, const int32_t* kv_off, const int32_t* prefix_len,
                   int32_t B, int32_t n_layers, int32_t n_heads, int32_t head_dim,
                   int32_t s_pool, int32_t dtype, int32_t* new_len, void* stream);

/* The whole verify step: embedding of tok, n_layers x {RMSNorm, QKV, rotary at
 * position prefix_len + depth, tree K/V written to the pool, tree attention, output
 * projection + residual, RMSNorm, SwiGLU FFN + residual}, final RMSNorm, LM head,
 * greedy argmax, longest accepted path, compaction.  logits ([T][vocab] fp32) may be
 * NULL when only the predictions are wanted: in bf16 mode the argmax is then taken in
 * the LM head's epilogue and no logits are ever written to memory (same predictions,
 * bit for bit, as with a logits buffer); in fp32 mode they are kept in the workspace.
 * All other outputs as in accept_path / kv_compact. */
int32_t tr_verify_step(const trj_model_desc* desc, const trj_weights* weights, void* k_pool,
                       void* v_pool, size_t kv_layer_stride, int32_t s_pool,
                       const int32_t* tok, const int32_t* parent, const int32_t* node_off,
                       const int32_t* kv_off, const int32_t* prefix_len, int32_t B, int32_t T,
                       int32_t max_seq_slots, void* workspace, size_t ws_bytes, float* logits,
                       int32_t* argmax_out, int32_t* accept_len, int32_t* best_node,
                       int32_t* path, int32_t* bonus_tok, int32_t* new_len,
                       int32_t* status_dev, void* stream);

/* ---- Static tree template (appendix "Templates for Token Tree": one fixed sparse tree is
 * used for every verification step).  What depends on the tree alone is computed once
 * into a caller-owned device buffer: validity, depth and ancestor bit rows of every node,
 * and the rotary table cos/sin(p * theta^(-2j/head_dim)) for positions p = 0..max_pos-1.
 * tr_verify_step_template is tr_verify_step with that buffer: per step only the parts
 * that depend on the prefix lengths are recomputed (slot range checks, slot and position
 * of every row, the attention work list), in one launch, and results are identical.
 *  - tr_template_bytes: size of the buffer for B sequences, T rows, max_pos positions.
 *  - tr_template_prepare: fills it from parent[T] / node_off[B+1] (same meaning as in
 *    tr_verify_step).  A malformed tree is recorded in the buffer and marks its sequence
 *    (status_dev[s] = 1) in every step that uses it.
 *  - tr_verify_step_template: B, T, max_pos, the model's head_dim and node_off[] must be
 *    those the buffer was prepared with, and parent[] must hold the same tree (it is
 *    still read by the acceptance rule); a buffer prepared for other sizes or row
 *    ranges marks every affected sequence malformed instead of being used.  Every
 *    sequence needs prefix_len[s] + N_s <= max_pos, else it is marked as well.  The
 *    buffer is only read; several steps (and streams) may share it. */
int32_t tr_template_bytes(const trj_model_desc* desc, int32_t B, int32_t T, int32_t max_pos,
                          size_t* h_bytes);
int32_t tr_template_prepare(const trj_model_desc* desc, const int32_t* parent,
                            const int32_t* node_off, int32_t B, int32_t T, int32_t max_pos,
                            void* tmpl, size_t tmpl_bytes, void* stream);
int32_t tr_verify_step_template(const trj_model_desc* desc, const trj_weights* weights,
                                void* k_pool, void* v_pool, size_t kv_layer_stride, int32_t s_pool,
                                const int32_t* tok, const int32_t* parent, const int32_t* node_off,
                                const int32_t* kv_off, const int32_t* prefix_len, int32_t B,
                                int32_t T, int32_t max_seq_slots, const void* tmpl,
                                size_t tmpl_bytes, int32_t max_pos, void* workspace,
                                size_t ws_bytes, float* logits, int32_t* argmax_out,
                                int32_t* accept_len, int32_t* best_node, int32_t* path,
                                int32_t* bonus_tok, int32_t* new_len, int32_t* status_dev,
                                void* stream);

/* ---- TR-Jacobi decoding loop (section "TR-Jacobi Decoding") -------------------------
 * Generation starts from a tree whose nodes are ahead noise (Eq. 4), every round
 * verifies the tree with tr_verify_step's forward, commits the longest accepted path
 * plus the greedy token after it, and refills the tree from the predictions made below
 * the accepted node; one chain below the root carries tokens retrieved by prompt lookup
 * (paragraph "Retrieval-Augmented Jacobi Decoding").  The committed tokens equal plain
 * greedy decoding whatever the drafts are.
 *
 * Refill rule (the paper only says "the path's subsequent predictions"): the new tree
 * is laid over the old one with its root on the accepted node; a new node that is the
 * k-th child (index order) of its parent lies on the k-th child of the old node under
 * its parent, if there is one, and takes the prediction made there as its token; a new
 * node that lies on nothing takes ahead noise: ctx[r mod ctx_len] with r the
 * (step * TRJ_N_MAX + node + 1)-th SplitMix64 output for `seed` and ctx all committed
 * tokens.  The last retrieval_len nodes of the template must be a chain below the root;
 * prompt lookup tries suffix lengths max_ngram..1 of ctx, takes the most recent earlier
 * occurrence and copies up to retrieval_len following tokens over that chain.
 *
 * The four helpers below are pure host functions (no GPU is touched). */
typedef struct {
  int32_t n_nodes;         /* N, root included, 1..TRJ_N_MAX */
  const int32_t* h_parent; /* HOST [N]: parent[0] = -1, 0 <= parent[i] < i */
  int32_t retrieval_len;   /* R in 0..N-1 */
  int32_t max_ngram;       /* >= 1 */
  int32_t max_new_tokens;  /* >= 1 */
  int32_t eos_token;       /* generation stops after this token (kept); -1: never */
  uint64_t seed;
} trj_decode_config;

/* k-th output (k >= 1) of SplitMix64 started at state `seed`. */
uint64_t trj_splitmix64(uint64_t seed, uint64_t k);
int32_t trj_ahead_noise(const int32_t* h_ctx, int32_t ctx_len, uint64_t seed, int32_t step,
                        int32_t node, int32_t* h_token);
/* h_out[0..*h_found) = the retrieved tokens, *h_found <= r. */
int32_t trj_prompt_lookup(const int32_t* h_ctx, int32_t ctx_len, int32_t max_ngram, int32_t r,
                          int32_t* h_out, int32_t* h_found);
/* Tokens of the tree verified in round `step`; ctx's last token is the root.
 * h_argmax == NULL: first tree (all noise + lookup); else the previous round's
 * predictions [N] and accepted node `best`. */
int32_t trj_fill_tree(const int32_t* h_parent, int32_t n_nodes, int32_t retrieval_len,
                      const int32_t* h_ctx, int32_t ctx_len, int32_t max_ngram, uint64_t seed,
                      int32_t step, const int32_t* h_argmax, int32_t best, int32_t* h_tok);

/* Device scratch tr_jacobi_generate needs for these sizes and this pool capacity. */
int32_t tr_jacobi_generate_workspace_bytes(const trj_model_desc* desc, int32_t n_nodes,
                                           int32_t prompt_len, int32_t max_new_tokens,
                                           int32_t s_pool, size_t* h_bytes);

/* Greedy generation for ONE sequence whose K/V live at slot 0.. of the pool (kv offset
 * 0; s_pool slots per head, a multiple of TRJ_KV_BLOCK, at least prompt_len +
 * max_new_tokens + N).  The prompt's K/V are computed first by chain-shaped trees of
 * TRJ_N_MAX tokens (an ordinary causal forward), up to eight of them packed into one step
 * as "sequences" that share the K/V region; the pool's previous contents are ignored.  h_prompt: HOST [prompt_len], prompt_len >= 1, ids in [0, vocab).  Outputs
 * (HOST): h_tokens[max_new_tokens], *h_n_tokens, h_accept_hist[max_new_tokens] (accepted
 * drafts per round, may be NULL), *h_n_steps (rounds).  Synchronous: returns after the
 * stream has drained.  Errors as above; nothing is written to the host outputs'
 * token area on an argument error. */
int32_t tr_jacobi_generate(const trj_model_desc* desc, const trj_weights* weights, void* k_pool,
                           void* v_pool, size_t kv_layer_stride, int32_t s_pool,
                           const int32_t* h_prompt, int32_t prompt_len,
                           const trj_decode_config* cfg, void* workspace, size_t ws_bytes,
                           int32_t* h_tokens, int32_t* h_n_tokens, int32_t* h_accept_hist,
                           int32_t* h_n_steps, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TRJACOBI_H */
