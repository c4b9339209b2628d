// Internal launcher declarations shared by the .hip files.  Every launcher only
// enqueues on the given stream and returns a trj_status.
#pragma once
#include "common.h"

namespace trj {

struct Tunables {
  int gemm_target_wgs = 256;   // split-k is raised until a GEMM has this many workgroups
  int max_split_k = 8;
  int gemm_cfg = 0;            // 0: choose the workgroup shape per GEMM; 1..4 force one
  int gemm_big_t = 256;        // padded token rows from which wavefronts own two row tiles (0: never)
  int attn_target_wgs = 256;   // attention workgroups per launch aimed at (one per CU)
  int gemm_big_wt = 0;         // row tiles per wavefront of the many-rows kernel (2, 4; 0 = choose)
  int attn_xchg_min_blocks = 48;  // blocks per workgroup from which wavefront pairs split their loads
  int attn_min_bpw = 0;        // 32-slot blocks per wavefront, at least (0: 1 for trees of up to 64 nodes, else 2)
};
// trj_set_tunable writes the process-wide set; every entry point copies it once on entry
// (TuneScope) and every launch plan of that call, on that thread, reads the copy, so the
// workspace a call carves and the launches it makes always come from the same values.
const Tunables& tune();
struct TuneScope {
  Tunables snap;
  const Tunables* prev;
  TuneScope();
  ~TuneScope();
};

// per-kernel timing hooks (api.hip): when kernel class `cls` is being profiled, a HIP
// event is recorded on the stream before and after the launch
enum KernelClass {
  KC_NONE = 0, KC_GEMM_QKV = 1, KC_ATTN = 2, KC_ATTN_COMBINE = 3, KC_GEMM_O = 4,
  KC_REDUCE_NORM = 5, KC_GEMM_GATE_UP = 6, KC_GEMM_DOWN = 7, KC_GEMM_LM = 8, KC_ARGMAX = 9,
  KC_ACCEPT = 10, KC_KV_COMPACT = 11, KC_SETUP = 12
};
void prof_begin(int cls, hipStream_t st);
void prof_end(int cls, hipStream_t st);
struct ProfScope {
  int cls;
  hipStream_t st;
  ProfScope(int c, hipStream_t s) : cls(c), st(s) { prof_begin(cls, st); }
  ~ProfScope() { prof_end(cls, st); }
};

// tree_kernels.hip
int launch_tree_prep(const int32_t* parent, const int32_t* node_off, const int32_t* kv_off,
                     const int32_t* prefix_len, int B, int T, int s_pool, int max_seq_slots,
                     int32_t* depth, uint64_t* anc, int32_t* status_dev, int32_t* row_slot, int32_t* row_pos,
                     int32_t* row_seq, void* zero, size_t zero_bytes, hipStream_t st);
// List of the (sequence, key split, query group) triples that exist, for the bf16 attention
// launch: n records of 8 words {sequence, group, first row, rows, prefix length,
// kv_off / 32, split, 1 if the sequence has more than one group}, sequences ordered by length (prefix + tree), longest first, when
// B <= 1024 (else in index order); word 8 * B * qg_max * nsplit_max holds n.  Sequences
// whose status is not 0 are left out.  Must follow launch_tree_prep on the stream.
#define ATTN_ITEM_WORDS(B, qg_max, nsplit_max) ((size_t)(B) * (qg_max) * (nsplit_max) * 8 + 8)
int launch_attn_items(const int32_t* node_off, const int32_t* prefix_len, const int32_t* kv_off,
                      const int32_t* status_dev, int B, int rows_per_item, int qg_max,
                      int blocks_per_item, int nsplit_max, int32_t* items, hipStream_t st);
// A prepared tree template (device pointers into the caller's buffer): what depends on the
// tree alone.  hdr: 8 words {magic, B, T, head_dim, max_pos}; tstatus[B]: 1 = malformed tree;
// tnoff[B+1]: the row ranges it was made for; tseq[T]: row -> sequence (-1: none);
// cs[max_pos][head_dim/2]: cos, sin of position * theta^(-2j/head_dim).
struct TemplateView {
  int32_t* hdr;
  int32_t* depth;
  uint64_t* anc;
  int32_t* tstatus;
  int32_t* tnoff;
  int32_t* tseq;
  float2* cs;
};
int launch_template_prepare(const int32_t* parent, const int32_t* node_off, int B, int T, int dh,
                            int max_pos, float theta, const TemplateView& v, hipStream_t st);
// Everything a step needs besides the template: slot checks (status_dev), slot / position /
// sequence of every row, the bf16 attention work list (items may be null), zero fill.
int launch_template_step_prep(const TemplateView& v, const int32_t* node_off, const int32_t* kv_off,
                              const int32_t* prefix_len, int B, int T, int dh, int max_pos, int s_pool,
                              int max_seq_slots, int32_t* status_dev, int32_t* row_slot,
                              int32_t* row_pos, int32_t* row_seq, int rows_per_item, int qg_max,
                              int blocks_per_item, int nsplit_max, int32_t* items, void* zero,
                              size_t zero_bytes, hipStream_t st);
int launch_argmax(const float* logits, int T, int V, int32_t* out, hipStream_t st);
int launch_accept(const int32_t* argmax, const int32_t* tok, const int32_t* parent,
                  const int32_t* node_off, const int32_t* status_in, int B, int T,
                  int32_t* accept_len, int32_t* best_node, int32_t* path, int32_t* bonus_tok,
                  int32_t* status_dev, hipStream_t st);
int launch_kv_compact(void* k_pool, void* v_pool, size_t layer_stride, const int32_t* path,
                      const int32_t* accept_len, const int32_t* kv_off, const int32_t* prefix_len,
                      int B, int n_layers, int n_heads, int dh, int s_pool, int dtype,
                      int32_t* new_len, hipStream_t st);
int launch_kv_convert(void* k_pool, void* v_pool, void* k_plain, void* v_plain, int n_heads,
                      int dh, int s_pool, int slot0, int n_slots, int dtype, bool pack,
                      hipStream_t st);
int launch_pack_weight(void* dst, const void* src, int n_out, int n_in, int dtype, int kind,
                       int n_heads, int dh, hipStream_t st);

// f32_kernels.hip
int launch_rope_table(const int32_t* row_pos, int T, int dh, float theta, float2* cs,
                      hipStream_t st);
int launch_embed(const void* embed, const int32_t* tok, int T, int d, int vocab, int dtype,
                 float* x, hipStream_t st);
int launch_rmsnorm_f32(const float* x, const float* g, int T, int d, float eps, float* h,
                       hipStream_t st);
int launch_gemm_f32(const float* x, const float* w, int T, int n_in, int n_out, int add_to,
                    float* y, hipStream_t st);
int launch_rope_kv_f32(const float* qkv, const float2* cs, const int32_t* cs_row,
                       const int32_t* row_slot, int T,
                       int n_heads, int n_kv_heads, int dh, int s_pool, float* q, float* k_layer,
                       float* v_layer, hipStream_t st);
int launch_silu_mul_f32(const float* gu, int T, int F, float* act, hipStream_t st);
int launch_tree_attn_f32(const float* q, const float* k_layer, const float* v_layer,
                         const uint64_t* anc, const int32_t* row_seq, const int32_t* node_off,
                         const int32_t* kv_off, const int32_t* prefix_len,
                         const int32_t* status_dev, int T, int n_heads, int n_kv_heads, int dh,
                         int s_pool, int max_slots, float scale, float* out, hipStream_t st);

// gemm_bf16.hip
// RMSNorm with the division deferred to the consumer: the producer of the activations
// writes bf16(x * g) (not yet divided by the row's norm) and, per row, partial sums of x^2
// over `parts` column parts; a projection of those activations multiplies its accumulators
// by 1 / sqrt(mean(x^2) + eps) of the token row before its epilogue.  (x*g*inv and (x*g)*inv
// round to bf16 with the same relative error, and the product with W is linear in inv.)
// The producer then needs no row-wide reduction and spreads over the whole chip.
constexpr int RS_MAX_PARTS = 4;
struct RowScale {
  const float* ssq;  // [parts][tp]; nullptr: activations are used as they are
  int parts, tp;
  float inv_d, eps;
};
int reduce_norm_parts(int d);
int gemm_bf16_split_k(int n_out, int tp, int n_in);
int gemm_bf16_clamp_split(int n_out, int tp, int n_in, int split_k);
void gemm_bf16_describe_plan(int tp, int n_in, int n_out, int split_k, int32_t out[6]);
int launch_gemm_store_f32(const uint16_t* xp, const uint16_t* w, int T, int tp, int n_in,
                          int n_out, int split_k, const RowScale& rs, float* y, hipStream_t st);
size_t gemm_lm_argmax_scratch_bytes(int T, int n_out);
int launch_gemm_lm_argmax(const uint16_t* xp, const uint16_t* w, int T, int tp, int n_in, int n_out,
                          const RowScale& rs, void* cand, int32_t* argmax_out, hipStream_t st);
int launch_gemm_gate_up(const uint16_t* xp, const uint16_t* w, int tp, int n_in, int d_ffn,
                        const RowScale& rs, uint16_t* act, hipStream_t st);
int launch_gemm_qkv(const uint16_t* xp, const uint16_t* w, int T, int tp, int n_in, int n_heads,
                    int n_kv_heads, int dh, int s_pool, const RowScale& rs, const float2* cs,
                    const int32_t* cs_row, const int32_t* row_slot, uint16_t* q, uint16_t* k_layer,
                    uint16_t* v_layer, hipStream_t st);
// x[t] = E[tok[t]] (fp32), or x[t] += the split-k partial sums; hp = bf16(x * g) tiled and the
// rows' partial sums of squares for the consumer's RowScale, one launch
int launch_embed_norm(const uint16_t* embed, const int32_t* tok, int T, int d, int vocab, float* x,
                      const float* g, int tp, uint16_t* hp, float* ssq, hipStream_t st);
int launch_reduce_norm(const float* partial, int n_split, float* x, const float* g, int T, int d,
                       int tp, uint16_t* hp, float* ssq, hipStream_t st);
int launch_sum_splits(const float* partial, int n_split, size_t n, float* y, hipStream_t st);
int launch_tile_activation(const uint16_t* x, int T, int n, int tp, uint16_t* xp, hipStream_t st);

// attn_bf16.hip
void attn_bf16_plan(int B, int T, int n_heads, int max_seq_slots, int* ntw, int* qg_max, int* bpwg,
                    int* nsplit_max);
size_t attn_bf16_ws_floats(int B, int tiles_per_seq, int n_heads, int dh, int nsplit_max);
int launch_zero_bytes(void* p, size_t bytes, hipStream_t st);
int launch_tree_attn_bf16(const uint16_t* q, const uint16_t* k_layer, const uint16_t* v_layer,
                          const uint64_t* anc, const int32_t* node_off,
                          const int32_t* kv_off, const int32_t* prefix_len,
                          const int32_t* status_dev, const int32_t* items, int B, int T,
                          int n_heads, int n_kv_heads, int dh, int s_pool, int max_seq_slots,
                          float scale, float* ws, int tiled, int tp, uint16_t* out, hipStream_t st);

// api.hip: the forward pass behind tr_verify_step (with_head == false: decoder layers
// only, for prompt passes), its workspace need, and the model-descriptor check
int step_impl(const trj_model_desc* desc, const trj_weights* weights, void* k_pool, void* v_pool,
              size_t kv_layer_stride, int32_t s_pool, const int32_t* tok, const int32_t* parent,
              const int32_t* node_off, const int32_t* kv_off, const int32_t* prefix_len,
              int32_t B, int32_t T, int32_t max_seq_slots, void* workspace, size_t ws_bytes,
              float* logits, int32_t* argmax_out, int32_t* accept_len, int32_t* best_node,
              int32_t* path, int32_t* bonus_tok, int32_t* new_len, int32_t* status_dev,
              bool with_head, hipStream_t st, const TemplateView* tmpl = nullptr, int max_pos = 0);
size_t template_carve(void* base, int B, int T, int dh, int max_pos, TemplateView* v);
size_t step_workspace_bytes(const trj_model_desc& m, int B, int T, int max_seq_slots);
int check_model(const trj_model_desc* m);

// token rows are padded to whole 32-row MFMA tiles: 1, 2, 3 or 4 tiles per workgroup pass,
// beyond that blocks of 4
inline int padded_rows(int T) { return T <= 96 ? (T <= 32 ? 32 : (T + 31) / 32 * 32) : (T + 127) / 128 * 128; }

}  // namespace trj
