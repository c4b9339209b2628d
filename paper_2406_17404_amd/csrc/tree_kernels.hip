// Integer / byte kernels of the verify step: tree bookkeeping (depth, ancestor bit
// rows), greedy argmax, longest accepted path, KV compaction, and the layout
// converters.  All results here are exact (no floating point decides anything except
// the comparisons inside argmax).
#include "common.h"
#include "kernels.h"

namespace trj {

// ------------------------------------------------------------------ tree bookkeeping
// One workgroup of TRJ_N_MAX threads per sequence.  A tree is well formed when
// parent[0] == -1 and 0 <= parent[i] < i; then walking parents strictly decreases the
// index, so every walk ends at the root.  When the KV arrays are given, the sequence's
// slot range must also lie inside the pool, start on a block boundary and hold at most
// max_seq_slots slots (the bound the host sized its launches and scratch with).  Rows of a
// malformed sequence get depth 0, empty bit rows and row_slot -1, which makes every
// later kernel skip them.
__global__ void fill_i32_kernel(int32_t* p, int32_t v, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

__global__ __launch_bounds__(TRJ_N_MAX) void tree_prep_kernel(
    const int32_t* __restrict__ parent, const int32_t* __restrict__ node_off,
    const int32_t* __restrict__ kv_off, const int32_t* __restrict__ prefix_len, int T, int s_pool,
    int max_seq_slots, int32_t* __restrict__ depth, uint64_t* __restrict__ anc, int32_t* __restrict__ status_dev,
    int32_t* __restrict__ row_slot, int32_t* __restrict__ row_pos, int32_t* __restrict__ row_seq) {
  __shared__ int32_t par[TRJ_N_MAX];
  __shared__ int32_t bad;
  const int s = blockIdx.x, i = threadIdx.x;
  int r0 = node_off[s], r1 = node_off[s + 1];
  // row range must lie inside [0, T] and hold 1..TRJ_N_MAX rows
  bool range_ok = r0 >= 0 && r1 <= T && r1 > r0 && (r1 - r0) <= TRJ_N_MAX;
  int n = range_ok ? r1 - r0 : 0;
  if (i == 0) {
    int b = range_ok ? 0 : 1;
    if (kv_off && range_ok) {
      int ko = kv_off[s], L = prefix_len[s];
      if (ko < 0 || (ko & (TRJ_KV_BLOCK - 1)) || L < 0 || (long)ko + L + n > (long)s_pool ||
          (long)L + n > (long)max_seq_slots)
        b = 1;
    }
    bad = b;
  }
  __syncthreads();
  if (i < n) {
    int p = parent[r0 + i];
    par[i] = p;
    if (i == 0 ? p != -1 : (p < 0 || p >= i)) atomicOr(&bad, 1);
  }
  __syncthreads();
  const int is_bad = bad;
  if (i == 0) status_dev[s] = is_bad;
  if (i >= n) return;  // nothing is written outside a valid row range
  uint64_t lo = 0, hi = 0;
  int d = 0;
  if (!is_bad) {
    d = -1;
    for (int j = i; j >= 0; j = par[j]) {
      if (j < 64) lo |= 1ull << j; else hi |= 1ull << (j - 64);
      ++d;
    }
  }
  depth[r0 + i] = d;
  anc[2 * (size_t)(r0 + i)] = lo;
  anc[2 * (size_t)(r0 + i) + 1] = hi;
  if (row_slot) {
    int L = prefix_len[s];
    row_slot[r0 + i] = is_bad ? -1 : kv_off[s] + L + i;
    row_pos[r0 + i] = is_bad ? 0 : L + d;
    row_seq[r0 + i] = is_bad ? -1 : s;
  }
}

// rows that no valid sequence covers must read as "skip": one launch clears all five arrays,
// and a further buffer of the caller's (the attention output, whose padding rows and rows of
// malformed sequences must read as zeros)
__global__ void prep_clear_kernel(int32_t* depth, int32_t* anc_words, int32_t* row_slot,
                                  int32_t* row_pos, int32_t* row_seq, int T, uint32_t* zero,
                                  size_t zero_words) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < zero_words) zero[i] = 0;
  if (i < (size_t)4 * T) anc_words[i] = 0;
  if (i < T) {
    depth[i] = 0;
    if (row_slot) {
      row_slot[i] = -1;
      row_pos[i] = 0;
      row_seq[i] = -1;
    }
  }
}

// One workgroup of 1024 threads builds the attention launch's item list.  Chunks of 1024
// sequences: thread i owns sequence base + i, counts its items (query groups x key splits
// of blocks_per_item 32-slot blocks; 0 when its status is not 0), and an inclusive scan
// over the chunk gives every sequence its place.  With one
// chunk (B <= 1024) the sequences are first ranked by length, longest first (ties by
// index), so that the long ones start early and the launch ends evenly.
__device__ inline void attn_items_body(
    const int32_t* __restrict__ node_off, const int32_t* __restrict__ prefix_len,
    const int32_t* __restrict__ kv_off, const int32_t* __restrict__ status, int B,
    int rows_per_item, int qg_max, int blocks_per_item, int nsplit_max,
    int32_t* __restrict__ items, int32_t* key, int32_t* cnt, int32_t* scan) {
  const int tid = threadIdx.x;
  int carry = 0;
  for (int base = 0; base < B; base += 1024) {
    const int s = base + tid;
    int n = 0, len = -1;
    if (s < B && status[s] == 0) {
      n = node_off[s + 1] - node_off[s];
      len = prefix_len[s] + n;
    }
    int ng = (n + rows_per_item - 1) / rows_per_item;
    if (ng > qg_max) ng = qg_max;
    int nsp = (((len + 31) >> 5) + blocks_per_item - 1) / blocks_per_item;
    if (nsp > nsplit_max) nsp = nsplit_max;
    const int nq = len < 0 ? 0 : ng * nsp;
    int place = tid;  // position of this sequence within the chunk
    if (B <= 1024) {
      key[tid] = len;
      __syncthreads();
      place = 0;
      for (int j = 0; j < B; ++j) place += key[j] > len || (key[j] == len && j < tid);
    }
    __syncthreads();
    if (s < B) cnt[place] = nq;
    else if (tid >= B - base) cnt[tid] = 0;
    __syncthreads();
    scan[tid] = cnt[tid];
    __syncthreads();
    for (int d = 1; d < 1024; d <<= 1) {
      int v = tid >= d ? scan[tid - d] : 0;
      __syncthreads();
      scan[tid] += v;
      __syncthreads();
    }
    if (s < B) {
      const int at = carry + scan[place] - nq;
      for (int j = 0; j < nq; ++j) {  // the query groups of a split next to each other
        int32_t* rec = items + (size_t)(at + j) * 8;
        rec[0] = s;
        rec[1] = j % ng;
        rec[2] = node_off[s];
        rec[3] = n;
        rec[4] = len - n;
        rec[5] = kv_off[s] >> 5;
        rec[6] = j / ng;
        rec[7] = ng > 1;  // another query group of the sequence reads the same blocks
      }
    }
    carry += scan[1023];
    __syncthreads();
  }
  if (tid == 0) items[(size_t)B * qg_max * nsplit_max * 8] = carry;
}

__global__ __launch_bounds__(1024) void attn_items_kernel(
    const int32_t* __restrict__ node_off, const int32_t* __restrict__ prefix_len,
    const int32_t* __restrict__ kv_off, const int32_t* __restrict__ status, int B,
    int rows_per_item, int qg_max, int blocks_per_item, int nsplit_max,
    int32_t* __restrict__ items) {
  __shared__ int32_t key[1024], cnt[1024], scan[1024];
  attn_items_body(node_off, prefix_len, kv_off, status, B, rows_per_item, qg_max, blocks_per_item,
                  nsplit_max, items, key, cnt, scan);
}

int launch_attn_items(const int32_t* node_off, const int32_t* prefix_len, const int32_t* kv_off,
                      const int32_t* status_dev, int B, int rows_per_item, int qg_max,
                      int blocks_per_item, int nsplit_max, int32_t* items, hipStream_t st) {
  if (qg_max < 1 || rows_per_item < 1 || blocks_per_item < 1 || nsplit_max < 1) return TRJ_ERR_BAD_SHAPE;
  attn_items_kernel<<<1, 1024, 0, st>>>(node_off, prefix_len, kv_off, status_dev, B, rows_per_item,
                                        qg_max, blocks_per_item, nsplit_max, items);
  return check_launch();
}

int launch_tree_prep(const int32_t* parent, const int32_t* node_off, const int32_t* kv_off,
                     const int32_t* prefix_len, int B, int T, int s_pool, int max_seq_slots,
                     int32_t* depth, uint64_t* anc, int32_t* status_dev, int32_t* row_slot, int32_t* row_pos,
                     int32_t* row_seq, void* zero, size_t zero_bytes, hipStream_t st) {
  const size_t zw = zero ? zero_bytes / 4 : 0, n = zw > (size_t)4 * T ? zw : (size_t)4 * T;
  prep_clear_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(
      depth, reinterpret_cast<int32_t*>(anc), row_slot, row_pos, row_seq, T,
      static_cast<uint32_t*>(zero), zw);
  tree_prep_kernel<<<B, TRJ_N_MAX, 0, st>>>(parent, node_off, kv_off, prefix_len, T, s_pool,
                                            max_seq_slots, depth, anc, status_dev, row_slot, row_pos, row_seq);
  return check_launch();
}

// ------------------------------------------------------------------ static tree template
// The paper verifies with ONE fixed sparse tree in every step (appendix "Templates for
// Token Tree"), so everything that depends on the tree alone is computed once into a
// caller-owned buffer: validity, depth and ancestor bits of every row, the row -> sequence
// map, and the rotary table over positions 0..max_pos-1.  A step then needs one small
// kernel for what depends on the prefix lengths: slot range checks, slot and position of
// every row, the attention launch's work list, and the zero fill of the step's padding.
constexpr int32_t TMPL_MAGIC = 0x54724a54;

__global__ void tmpl_finish_kernel(const int32_t* __restrict__ node_off, int B, int T, int dh,
                                   int max_pos, const int32_t* __restrict__ tstatus,
                                   int32_t* __restrict__ hdr, int32_t* __restrict__ tnoff,
                                   int32_t* __restrict__ tseq) {
  // one workgroup per sequence; tseq was cleared to -1 before
  const int s = blockIdx.x, i = threadIdx.x;
  if (s == 0 && i == 0) {
    hdr[0] = TMPL_MAGIC; hdr[1] = B; hdr[2] = T; hdr[3] = dh; hdr[4] = max_pos;
    hdr[5] = hdr[6] = hdr[7] = 0;
    tnoff[B] = node_off[B];
  }
  if (i == 0) tnoff[s] = node_off[s];
  if (tstatus[s] != 0) return;  // a malformed sequence owns no rows
  const int r0 = node_off[s], n = node_off[s + 1] - r0;
  if (i < n) tseq[r0 + i] = s;
}

int launch_template_prepare(const int32_t* parent, const int32_t* node_off, int B, int T, int dh,
                            int max_pos, float theta, const TemplateView& v, hipStream_t st) {
  int rc = launch_tree_prep(parent, node_off, nullptr, nullptr, B, T, 0, 0, v.depth, v.anc, v.tstatus,
                            nullptr, nullptr, nullptr, nullptr, 0, st);
  if (rc != TRJ_OK) return rc;
  fill_i32_kernel<<<(T + 255) / 256, 256, 0, st>>>(v.tseq, -1, T);
  tmpl_finish_kernel<<<B, TRJ_N_MAX, 0, st>>>(node_off, B, T, dh, max_pos, v.tstatus, v.hdr, v.tnoff,
                                              v.tseq);
  rc = check_launch();
  if (rc != TRJ_OK) return rc;
  return launch_rope_table(nullptr, max_pos, dh, theta, v.cs, st);
}

__global__ __launch_bounds__(1024) void tmpl_step_prep_kernel(
    TemplateView v, const int32_t* __restrict__ node_off, const int32_t* __restrict__ kv_off,
    const int32_t* __restrict__ prefix_len, int B, int T, int dh, int max_pos, int s_pool,
    int max_seq_slots, int32_t* __restrict__ status_dev, int32_t* __restrict__ row_slot,
    int32_t* __restrict__ row_pos, int32_t* __restrict__ row_seq, int rows_per_item, int qg_max,
    int blocks_per_item, int nsplit_max, int32_t* __restrict__ items, uint32_t* __restrict__ zero,
    size_t zero_words) {
  const int tid = threadIdx.x;
  if (blockIdx.x > 0) {  // the other workgroups clear the step's padding
    for (size_t i = (size_t)(blockIdx.x - 1) * 1024 + tid; i < zero_words;
         i += (size_t)(gridDim.x - 1) * 1024)
      zero[i] = 0;
    return;
  }
  __shared__ int32_t key[1024], cnt[1024], scan[1024];
  __shared__ int32_t hdr_bad;
  if (tid == 0)
    hdr_bad = !(v.hdr[0] == TMPL_MAGIC && v.hdr[1] == B && v.hdr[2] == T && v.hdr[3] == dh &&
                v.hdr[4] == max_pos);
  __syncthreads();
  for (int s = tid; s < B; s += 1024) {
    // the step's row ranges must be the template's (which were validated when it was made)
    bool ok = !hdr_bad && v.tstatus[s] == 0 && node_off[s] == v.tnoff[s] &&
              node_off[s + 1] == v.tnoff[s + 1];
    if (ok) {
      const int n = v.tnoff[s + 1] - v.tnoff[s];
      const int ko = kv_off[s], L = prefix_len[s];
      if (ko < 0 || (ko & (TRJ_KV_BLOCK - 1)) || L < 0 || (long)ko + L + n > (long)s_pool ||
          (long)L + n > (long)max_seq_slots || (long)L + n > (long)max_pos)
        ok = false;
    }
    status_dev[s] = ok ? 0 : 1;
  }
  __threadfence_block();
  __syncthreads();
  for (int t = tid; t < T; t += 1024) {
    const int s = hdr_bad ? -1 : v.tseq[t];
    const bool bad = s < 0 || s >= B || status_dev[s] != 0;
    const int L = bad ? 0 : prefix_len[s];
    row_slot[t] = bad ? -1 : kv_off[s] + L + (t - v.tnoff[s]);
    row_pos[t] = bad ? 0 : L + v.depth[t];
    row_seq[t] = bad ? -1 : s;
  }
  if (items) {
    __syncthreads();
    attn_items_body(node_off, prefix_len, kv_off, status_dev, B, rows_per_item, qg_max,
                    blocks_per_item, nsplit_max, items, key, cnt, scan);
  }
}

int launch_template_step_prep(const TemplateView& v, const int32_t* node_off, const int32_t* kv_off,
                              const int32_t* prefix_len, int B, int T, int dh, int max_pos, int s_pool,
                              int max_seq_slots, int32_t* status_dev, int32_t* row_slot,
                              int32_t* row_pos, int32_t* row_seq, int rows_per_item, int qg_max,
                              int blocks_per_item, int nsplit_max, int32_t* items, void* zero,
                              size_t zero_bytes, hipStream_t st) {
  const size_t zw = zero ? zero_bytes / 4 : 0;
  size_t zwgs = (zw + 16 * 1024 - 1) / (16 * 1024);  // 16 words per thread and pass
  if (zwgs > 512) zwgs = 512;
  tmpl_step_prep_kernel<<<(unsigned)(1 + zwgs), 1024, 0, st>>>(
      v, node_off, kv_off, prefix_len, B, T, dh, max_pos, s_pool, max_seq_slots, status_dev, row_slot,
      row_pos, row_seq, rows_per_item, qg_max, blocks_per_item, nsplit_max, items,
      static_cast<uint32_t*>(zero), zw);
  return check_launch();
}

// ------------------------------------------------------------------ greedy argmax
// One workgroup per row; lowest index wins ties; NaN never compares greater.
// One workgroup per row; every thread keeps ARGMAX_UNROLL 16-byte loads in flight (the row
// is read once, so the kernel is a latency chain unless the loads are batched).
constexpr int ARGMAX_THREADS = 1024, ARGMAX_UNROLL = 4;
__device__ inline void amax_merge(float& bv, int& bi, float v, int i) {
  if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
}
__global__ __launch_bounds__(ARGMAX_THREADS) void argmax_kernel(const float* __restrict__ logits,
                                                                int V, int32_t* __restrict__ out) {
  const float* row = logits + (size_t)blockIdx.x * V;
  float bv = -INFINITY;
  int bi = INT32_MAX;
  const int tid = threadIdx.x;
  if ((V & 3) == 0 && (((uintptr_t)row) & 15) == 0) {
    const float4* r4 = reinterpret_cast<const float4*>(row);
    const int n4 = V >> 2;
    for (int i0 = tid; i0 < n4; i0 += ARGMAX_THREADS * ARGMAX_UNROLL) {
      float4 x[ARGMAX_UNROLL];
#pragma unroll
      for (int u = 0; u < ARGMAX_UNROLL; ++u) x[u] = r4[min(i0 + u * ARGMAX_THREADS, n4 - 1)];
#pragma unroll
      for (int u = 0; u < ARGMAX_UNROLL; ++u) {
        const int i = i0 + u * ARGMAX_THREADS;
        if (i < n4) {
          amax_merge(bv, bi, x[u].x, 4 * i);
          amax_merge(bv, bi, x[u].y, 4 * i + 1);
          amax_merge(bv, bi, x[u].z, 4 * i + 2);
          amax_merge(bv, bi, x[u].w, 4 * i + 3);
        }
      }
    }
  } else {
    for (int i = tid; i < V; i += ARGMAX_THREADS) amax_merge(bv, bi, row[i], i);
  }
  for (int o = 32; o > 0; o >>= 1) {
    float ov = __shfl_xor(bv, o);
    int oi = __shfl_xor(bi, o);
    amax_merge(bv, bi, ov, oi);
  }
  __shared__ float sv[ARGMAX_THREADS / WAVE];
  __shared__ int si[ARGMAX_THREADS / WAVE];
  if ((tid & 63) == 0) { sv[tid >> 6] = bv; si[tid >> 6] = bi; }
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < ARGMAX_THREADS / WAVE; ++w) amax_merge(bv, bi, sv[w], si[w]);
    out[blockIdx.x] = bi == INT32_MAX ? 0 : bi;
  }
}

int launch_argmax(const float* logits, int T, int V, int32_t* out, hipStream_t st) {
  argmax_kernel<<<T, ARGMAX_THREADS, 0, st>>>(logits, V, out);
  return check_launch();
}

// ------------------------------------------------------------------ accept
// One workgroup of TRJ_N_MAX threads per sequence.  ok[i] is evaluated by walking from
// i to the root; best = max over ok nodes of (depth, -index).  status_in (optional)
// marks sequences an earlier kernel already found malformed.
__global__ __launch_bounds__(TRJ_N_MAX) void accept_kernel(
    const int32_t* __restrict__ argmax, const int32_t* __restrict__ tok,
    const int32_t* __restrict__ parent, const int32_t* __restrict__ node_off, int T,
    const int32_t* status_in, int32_t* __restrict__ accept_len,
    int32_t* __restrict__ best_node, int32_t* __restrict__ path, int32_t* __restrict__ bonus_tok,
    int32_t* status_dev) {  // status_in may alias status_dev
  __shared__ int32_t par[TRJ_N_MAX], tk[TRJ_N_MAX], am[TRJ_N_MAX];
  __shared__ int32_t bad, best_key;
  const int s = blockIdx.x, i = threadIdx.x;
  int r0 = node_off[s], r1 = node_off[s + 1];
  bool range_ok = r0 >= 0 && r1 <= T && r1 > r0 && (r1 - r0) <= TRJ_N_MAX;
  int n = range_ok ? r1 - r0 : 0;
  if (i == 0) {
    bad = (range_ok && !(status_in && status_in[s] != 0)) ? 0 : 1;
    best_key = -1;
  }
  __syncthreads();
  if (i < n) {
    int p = parent[r0 + i];
    par[i] = p;
    tk[i] = tok[r0 + i];
    am[i] = argmax[r0 + i];
    if (i == 0 ? p != -1 : (p < 0 || p >= i)) atomicOr(&bad, 1);
  }
  __syncthreads();
  int32_t* my_path = path + (size_t)s * TRJ_N_MAX;
  my_path[i] = -1;
  if (bad) {
    if (i == 0) {
      status_dev[s] = 1;
      accept_len[s] = -1;
      best_node[s] = -1;
      bonus_tok[s] = -1;
    }
    return;
  }
  if (i < n) {
    bool ok = true;
    int d = 0;
    for (int j = i; j > 0; j = par[j]) {
      ok = ok && (tk[j] == am[par[j]]);
      ++d;
    }
    if (ok) atomicMax(&best_key, (d << 8) | (255 - i));
  }
  __syncthreads();  // also orders the -1 fill above before the path writes below
  if (i == 0) {
    int key = best_key;  // the root is always ok, so key >= 255
    int b = 255 - (key & 255), d = key >> 8;
    status_dev[s] = 0;
    accept_len[s] = d;
    best_node[s] = b;
    bonus_tok[s] = am[b];
    for (int j = b, k = d; j >= 0; j = par[j], --k) my_path[k] = j;
  }
}

int launch_accept(const int32_t* argmax, const int32_t* tok, const int32_t* parent,
                  const int32_t* node_off, const int32_t* status_in, int B, int T,
                  int32_t* accept_len, int32_t* best_node, int32_t* path, int32_t* bonus_tok,
                  int32_t* status_dev, hipStream_t st) {
  accept_kernel<<<B, TRJ_N_MAX, 0, st>>>(argmax, tok, parent, node_off, T, status_in, accept_len,
                                         best_node, path, bonus_tok, status_dev);
  return check_launch();
}

// ------------------------------------------------------------------ KV compaction
// One workgroup per (sequence, layer*head) plane, one thread per head_dim column.
// Row j of the accepted path moves from slot base+path[j] to base+j.  path is
// increasing with path[j] >= j, so copying in increasing j with a barrier between rows
// never overwrites a row that is still to be read.
template <typename E>
__global__ void kv_compact_kernel(E* __restrict__ k_pool, E* __restrict__ v_pool,
                                  size_t layer_stride, const int32_t* __restrict__ path,
                                  const int32_t* __restrict__ accept_len,
                                  const int32_t* __restrict__ kv_off,
                                  const int32_t* __restrict__ prefix_len, int n_heads, int dh,
                                  int s_pool, int32_t* __restrict__ new_len) {
  const int s = blockIdx.x, plane = blockIdx.y;
  const int layer = plane / n_heads, head = plane % n_heads;
  const int a = accept_len[s];
  const int L = prefix_len[s];
  if (plane == 0 && threadIdx.x == 0) new_len[s] = a < 0 ? L : L + a + 1;
  if (a < 0 || L < 0 || kv_off[s] < 0) return;
  const int base = kv_off[s] + L;
  E* kp = k_pool + layer * layer_stride + (size_t)head * s_pool * dh;
  E* vp = v_pool + layer * layer_stride + (size_t)head * s_pool * dh;
  const int32_t* pth = path + (size_t)s * TRJ_N_MAX;
  for (int j = 0; j <= a && j < TRJ_N_MAX; ++j) {
    int src = pth[j];
    if (src > j && src < TRJ_N_MAX && base + src < s_pool) {  // uniform over the workgroup
      for (int c = threadIdx.x; c < dh; c += blockDim.x) {
        E kk = kp[k_off(base + src, c, dh)];
        E vv = vp[v_off(base + src, c, dh)];
        kp[k_off(base + j, c, dh)] = kk;
        vp[v_off(base + j, c, dh)] = vv;
      }
    }
    __syncthreads();
  }
}

int launch_kv_compact(void* k_pool, void* v_pool, size_t layer_stride, const int32_t* path,
                      const int32_t* accept_len, const int32_t* kv_off, const int32_t* prefix_len,
                      int B, int n_layers, int n_heads, int dh, int s_pool, int dtype,
                      int32_t* new_len, hipStream_t st) {
  dim3 grid(B, n_layers * n_heads);
  int threads = dh < 64 ? 64 : (dh > 256 ? 256 : dh);
  if (dtype == TRJ_BF16)
    kv_compact_kernel<uint16_t><<<grid, threads, 0, st>>>((uint16_t*)k_pool, (uint16_t*)v_pool,
                                                          layer_stride, path, accept_len, kv_off,
                                                          prefix_len, n_heads, dh, s_pool, new_len);
  else
    kv_compact_kernel<uint32_t><<<grid, threads, 0, st>>>((uint32_t*)k_pool, (uint32_t*)v_pool,
                                                          layer_stride, path, accept_len, kv_off,
                                                          prefix_len, n_heads, dh, s_pool, new_len);
  return check_launch();
}

// ------------------------------------------------------------------ layout converters
template <typename E, bool PACK>
__global__ void kv_convert_kernel(E* __restrict__ k_pool, E* __restrict__ v_pool,
                                  E* __restrict__ k_plain, E* __restrict__ v_plain, int dh,
                                  int s_pool, int slot0, int n_slots) {
  const int head = blockIdx.y;
  size_t total = (size_t)n_slots * dh;
  E* kp = k_pool + (size_t)head * s_pool * dh;
  E* vp = v_pool + (size_t)head * s_pool * dh;
  E* kl = k_plain + (size_t)head * n_slots * dh;
  E* vl = v_plain + (size_t)head * n_slots * dh;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (size_t)gridDim.x * blockDim.x) {
    int sl = (int)(i / dh), c = (int)(i % dh);
    if (PACK) {
      kp[k_off(slot0 + sl, c, dh)] = kl[i];
      vp[v_off(slot0 + sl, c, dh)] = vl[i];
    } else {
      kl[i] = kp[k_off(slot0 + sl, c, dh)];
      vl[i] = vp[v_off(slot0 + sl, c, dh)];
    }
  }
}

int launch_kv_convert(void* k_pool, void* v_pool, void* k_plain, void* v_plain, int n_heads,
                      int dh, int s_pool, int slot0, int n_slots, int dtype, bool pack,
                      hipStream_t st) {
  if (n_slots == 0) return TRJ_OK;
  size_t total = (size_t)n_slots * dh;
  int bx = (int)((total + 255) / 256);
  if (bx > 1024) bx = 1024;
  dim3 grid(bx, n_heads);
#define TRJ_KVC(E, P)                                                                         \
  kv_convert_kernel<E, P><<<grid, 256, 0, st>>>((E*)k_pool, (E*)v_pool, (E*)k_plain,          \
                                                (E*)v_plain, dh, s_pool, slot0, n_slots)
  if (dtype == TRJ_BF16) {
    if (pack) TRJ_KVC(uint16_t, true); else TRJ_KVC(uint16_t, false);
  } else {
    if (pack) TRJ_KVC(uint32_t, true); else TRJ_KVC(uint32_t, false);
  }
#undef TRJ_KVC
  return check_launch();
}

// one thread per 8-element granule of the packed matrix
template <typename E>
__global__ void pack_weight_kernel(E* __restrict__ dst, const E* __restrict__ src, int n_out,
                                   int n_in, int kind, int n_heads, int dh) {
  size_t granules = (size_t)n_out * (n_in >> 3);
  for (size_t g = (size_t)blockIdx.x * blockDim.x + threadIdx.x; g < granules;
       g += (size_t)gridDim.x * blockDim.x) {
    // granule g of the packed buffer: decode (tile row, k-step, half, row in tile)
    size_t tile = g >> 6;
    int lane = (int)(g & 63);
    int ksteps = n_in >> 4;
    int rt = (int)(tile / ksteps), ks = (int)(tile % ksteps);
    int r = rt * 32 + (lane & 31), k = ks * 16 + (lane >> 5) * 8;
    const E* s = src + (size_t)logical_row(r, kind, n_out, n_heads, dh) * n_in + k;
    E* d = dst + g * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) d[e] = s[e];
  }
}

int launch_pack_weight(void* dst, const void* src, int n_out, int n_in, int dtype, int kind,
                       int n_heads, int dh, hipStream_t st) {
  size_t granules = (size_t)n_out * (n_in >> 3);
  int bx = (int)((granules + 255) / 256);
  if (bx > 65536) bx = 65536;
  if (dtype == TRJ_BF16)
    pack_weight_kernel<uint16_t><<<bx, 256, 0, st>>>((uint16_t*)dst, (const uint16_t*)src, n_out,
                                                     n_in, kind, n_heads, dh);
  else
    pack_weight_kernel<uint32_t><<<bx, 256, 0, st>>>((uint32_t*)dst, (const uint32_t*)src, n_out,
                                                     n_in, kind, n_heads, dh);
  return check_launch();
}

}  // namespace trj
