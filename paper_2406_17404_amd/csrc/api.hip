// C-ABI entry points of libtrjacobi: argument checks, workspace carving and the order
// in which the kernels of the verify step are enqueued.  No arithmetic lives here.
#include <atomic>
#include <cstring>
#include <mutex>
#include <vector>

#include "../../include/trjacobi_dev.h"
#include "common.h"
#include "kernels.h"

namespace trj {

static Tunables g_tune;          // process-wide, written by trj_set_tunable under g_tune_mu
static std::mutex g_tune_mu;
static thread_local const Tunables* t_tune = nullptr;  // the running entry point's snapshot
const Tunables& tune() { return t_tune ? *t_tune : g_tune; }
TuneScope::TuneScope() : prev(t_tune) {
  if (prev) {
    snap = *prev;  // nested entry point: keep the outer call's values
  } else {
    std::lock_guard<std::mutex> lk(g_tune_mu);
    snap = g_tune;
  }
  t_tune = &snap;
}
TuneScope::~TuneScope() { t_tune = prev; }
static std::atomic<int> g_last_hip_error{0};
void note_hip_error(hipError_t e) { g_last_hip_error.store((int)e); }

// ---- optional per-kernel timing (trj_profile_begin / trj_profile_end)
struct Profiler {
  int cls = KC_NONE;       // class whose launch opens a timed span
  int cls_last = KC_NONE;  // class whose launch closes it (the same class: one launch)
  std::vector<hipEvent_t> start, stop;
  int used = 0;
  bool open = false;
};
static Profiler g_prof;
void prof_begin(int cls, hipStream_t st) {
  if (cls != g_prof.cls || g_prof.open || g_prof.used >= (int)g_prof.start.size()) return;
  (void)hipEventRecord(g_prof.start[g_prof.used], st);
  g_prof.open = true;
}
void prof_end(int cls, hipStream_t st) {
  if (cls != g_prof.cls_last || !g_prof.open) return;
  (void)hipEventRecord(g_prof.stop[g_prof.used++], st);
  g_prof.open = false;
}

// bump allocator over the caller's workspace; with base == nullptr it only measures
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* b) : base(static_cast<char*>(b)) {}
  template <typename T>
  T* take(size_t count) {
    off = align_up(off, 256);
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += count * sizeof(T);
    return p;
  }
};

struct TreeWs {
  int32_t *depth, *row_slot, *row_pos, *row_seq, *status;
  uint64_t* anc;
  float* attn;     // bf16 attention partials
  int32_t* items;  // bf16 attention work items and their count
  int attn_rows, attn_qg, attn_bpwg, attn_ns;  // the attention launch plan
};
struct StepWs {
  TreeWs t;
  float2* cs;
  float *x, *logits;
  void* cand;  // bf16 mode without logits: argmax candidates of the LM head's epilogue
  // bf16 mode
  uint16_t *hp, *q, *op, *act;
  float *partial, *ssq;
  // fp32 mode
  float *h, *qkv, *qf, *of, *gu, *actf;
};

static void carve_tree(Carver& c, int dtype, int B, int T, int H, int dh, int max_seq_slots,
                       TreeWs* w) {
  w->depth = c.take<int32_t>(T);
  w->row_slot = c.take<int32_t>(T);
  w->row_pos = c.take<int32_t>(T);
  w->row_seq = c.take<int32_t>(T);
  w->status = c.take<int32_t>(B);
  w->anc = c.take<uint64_t>(2 * (size_t)T);
  w->attn = nullptr;
  w->items = nullptr;
  w->attn_rows = w->attn_qg = w->attn_bpwg = w->attn_ns = 0;
  if (dtype == TRJ_BF16) {
    int ntw, qg, bpwg, ns;
    attn_bf16_plan(B, T, H, max_seq_slots, &ntw, &qg, &bpwg, &ns);
    w->attn = c.take<float>(attn_bf16_ws_floats(B, qg * ntw, H, dh, ns));
    w->items = c.take<int32_t>(ATTN_ITEM_WORDS(B, qg, ns));
    w->attn_rows = 32 * ntw;
    w->attn_qg = qg;
    w->attn_bpwg = bpwg;
    w->attn_ns = ns;
  }
}

static void carve_step(Carver& c, const trj_model_desc& m, int B, int T, int max_seq_slots,
                       bool need_logits, StepWs* w) {
  const int d = m.d_model, hd = m.n_heads * m.head_dim, F = m.d_ffn;
  const int kvd = (m.n_kv_heads ? m.n_kv_heads : m.n_heads) * m.head_dim;
  carve_tree(c, m.dtype, B, T, m.n_heads, m.head_dim, max_seq_slots, &w->t);
  w->cs = c.take<float2>((size_t)T * (m.head_dim / 2));
  w->x = c.take<float>((size_t)T * d);
  // without a logits buffer from the caller the fp32 mode keeps them here; the bf16 mode
  // takes the argmax in the LM head's epilogue and needs only its candidates
  w->logits = need_logits && m.dtype != TRJ_BF16 ? c.take<float>((size_t)T * m.vocab) : nullptr;
  w->cand = need_logits && m.dtype == TRJ_BF16
                ? c.take<char>(gemm_lm_argmax_scratch_bytes(T, m.vocab)) : nullptr;
  if (m.dtype == TRJ_BF16) {
    const int tp = padded_rows(T);
    w->hp = c.take<uint16_t>((size_t)tp * d);
    w->q = c.take<uint16_t>((size_t)T * hd);
    w->op = c.take<uint16_t>((size_t)tp * hd);
    w->act = c.take<uint16_t>((size_t)tp * F);
    int sk1 = gemm_bf16_split_k(d, tp, hd), sk2 = gemm_bf16_split_k(d, tp, F);
    w->partial = c.take<float>((size_t)(sk1 > sk2 ? sk1 : sk2) * T * d);
    w->ssq = c.take<float>((size_t)RS_MAX_PARTS * tp);
  } else {
    w->h = c.take<float>((size_t)T * d);
    w->qkv = c.take<float>((size_t)T * (hd + 2 * kvd));
    w->qf = c.take<float>((size_t)T * hd);
    w->of = c.take<float>((size_t)T * hd);
    w->gu = c.take<float>((size_t)T * 2 * F);
    w->actf = c.take<float>((size_t)T * F);
  }
}

static int check_desc(const trj_model_desc* m) {
  if (!m) return TRJ_ERR_NULLPTR;
  if (m->dtype != TRJ_F32 && m->dtype != TRJ_BF16) return TRJ_ERR_BAD_DTYPE;
  if (m->n_layers < 1 || m->d_model < 32 || m->n_heads < 1 || m->head_dim < 32 || m->d_ffn < 32 ||
      m->vocab < 32)
    return TRJ_ERR_BAD_SHAPE;
  // every projection's output width is a whole number of 32-row weight tiles (d_model for
  // the output and down projections, 2 * d_ffn in gate/up pairs of 16 + 16 rows)
  if ((m->d_model & 31) || (m->head_dim & 31) || (m->d_ffn & 31) || (m->vocab & 31))
    return TRJ_ERR_BAD_SHAPE;
  if (m->dtype == TRJ_BF16 && m->head_dim != 64 && m->head_dim != 128) return TRJ_ERR_BAD_SHAPE;
  if (m->dtype == TRJ_BF16 && m->d_model > 8192) return TRJ_ERR_BAD_SHAPE;
  if (!(m->rms_eps >= 0.f) || !(m->rope_theta > 0.f)) return TRJ_ERR_BAD_SHAPE;
  if (m->n_kv_heads < 0 || (m->n_kv_heads > 0 && m->n_heads % m->n_kv_heads != 0))
    return TRJ_ERR_BAD_SHAPE;
  return TRJ_OK;
}

static int check_batch(int B, int T, int s_pool, int max_seq_slots) {
  if (B < 1 || T < 1 || s_pool < TRJ_KV_BLOCK || (s_pool & (TRJ_KV_BLOCK - 1)))
    return TRJ_ERR_BAD_SHAPE;
  if (T < B) return TRJ_ERR_BAD_SHAPE;
  if ((long)T > (long)B * TRJ_N_MAX) return TRJ_ERR_TREE_TOO_LARGE;
  if (max_seq_slots < 1 || max_seq_slots > s_pool) return TRJ_ERR_BAD_SHAPE;
  return TRJ_OK;
}

#define TRJ_TRY(expr)          \
  do {                         \
    int rc_ = (expr);          \
    if (rc_ != TRJ_OK) return rc_; \
  } while (0)

}  // namespace trj

using namespace trj;

extern "C" {

const char* trj_version(void) { return "trjacobi 0.1 (gfx950)"; }
int32_t trj_last_hip_error(void) { return g_last_hip_error.load(); }

// Launch-shape knobs for experiments; values outside the range a launch plan can use are
// refused (a zero here would otherwise divide by zero in the plan).
int32_t trj_set_tunable(const char* name, int32_t value) {
  if (!name) return TRJ_ERR_NULLPTR;
  std::lock_guard<std::mutex> lk(g_tune_mu);
  const bool positive = value >= 1 && value <= (1 << 20);
  if (!strcmp(name, "gemm_target_wgs") && positive) g_tune.gemm_target_wgs = value;
  else if (!strcmp(name, "max_split_k") && positive) g_tune.max_split_k = value;
  else if (!strcmp(name, "gemm_cfg") && value >= 0 && value <= 6) g_tune.gemm_cfg = value;
  else if (!strcmp(name, "gemm_big_t") && value >= 0) g_tune.gemm_big_t = value;
  else if (!strcmp(name, "gemm_big_wt") && (value == 0 || value == 2 || value == 4)) g_tune.gemm_big_wt = value;
  else if (!strcmp(name, "attn_target_wgs") && positive) g_tune.attn_target_wgs = value;
  else if (!strcmp(name, "attn_min_bpw") && (positive || value == 0)) g_tune.attn_min_bpw = value;
  else if (!strcmp(name, "attn_xchg_min_blocks") && positive) g_tune.attn_xchg_min_blocks = value;
  else return TRJ_ERR_BAD_SHAPE;
  return TRJ_OK;
}

// Per-kernel timing: between trj_profile_begin and trj_profile_end every launch of the
// chosen kernel class is bracketed by HIP events on its stream (this is the one place
// where the library creates HIP objects: the events).  trj_profile_end waits for them and
// returns the durations in milliseconds.
int32_t trj_profile_begin_span(int32_t first_class, int32_t last_class, int32_t capacity);
int32_t trj_profile_begin(int32_t kernel_class, int32_t capacity) {
  return trj_profile_begin_span(kernel_class, kernel_class, capacity);
}
int32_t trj_profile_begin_span(int32_t kernel_class, int32_t last_class, int32_t capacity) {
  if (g_prof.cls != KC_NONE || kernel_class <= KC_NONE || kernel_class > KC_SETUP ||
      last_class <= KC_NONE || last_class > KC_SETUP || capacity < 1)
    return TRJ_ERR_BAD_SHAPE;
  g_prof.start.resize(capacity);
  g_prof.stop.resize(capacity);
  for (int i = 0; i < capacity; ++i) {
    hipError_t e1 = hipEventCreate(&g_prof.start[i]), e2 = hipEventCreate(&g_prof.stop[i]);
    if (e1 != hipSuccess || e2 != hipSuccess) {
      note_hip_error(e1 != hipSuccess ? e1 : e2);
      return TRJ_ERR_HIP;
    }
  }
  g_prof.used = 0;
  g_prof.open = false;
  g_prof.cls = kernel_class;
  g_prof.cls_last = last_class;
  return TRJ_OK;
}
int32_t trj_profile_end(float* h_ms, int32_t capacity, int32_t* h_count) {
  if (!h_ms || !h_count) return TRJ_ERR_NULLPTR;
  int rc = TRJ_OK;
  int n = g_prof.used < capacity ? g_prof.used : capacity;
  for (int i = 0; i < n; ++i) {
    hipError_t e = hipEventSynchronize(g_prof.stop[i]);
    if (e == hipSuccess) e = hipEventElapsedTime(&h_ms[i], g_prof.start[i], g_prof.stop[i]);
    if (e != hipSuccess) { note_hip_error(e); rc = TRJ_ERR_HIP; }
  }
  *h_count = n;
  for (size_t i = 0; i < g_prof.start.size(); ++i) {
    (void)hipEventDestroy(g_prof.start[i]);
    (void)hipEventDestroy(g_prof.stop[i]);
  }
  g_prof.start.clear();
  g_prof.stop.clear();
  g_prof.used = 0;
  g_prof.cls = KC_NONE;
  g_prof.cls_last = KC_NONE;
  g_prof.open = false;
  return rc;
}

int32_t trj_profile_event_overhead(int32_t pairs, float* h_avg_ms, void* stream) {
  if (!h_avg_ms) return TRJ_ERR_NULLPTR;
  if (pairs < 1 || pairs > 4096) return TRJ_ERR_BAD_SHAPE;
  hipStream_t st = (hipStream_t)stream;
  std::vector<hipEvent_t> ev(2 * (size_t)pairs);
  int rc = TRJ_OK;
  for (auto& e : ev)
    if (hipEventCreate(&e) != hipSuccess) rc = TRJ_ERR_HIP;
  if (rc == TRJ_OK) {
    for (int i = 0; i < pairs; ++i) {
      (void)hipEventRecord(ev[2 * i], st);
      (void)hipEventRecord(ev[2 * i + 1], st);
    }
    double sum = 0;
    for (int i = 0; i < pairs; ++i) {
      float ms = 0.f;
      hipError_t e = hipEventSynchronize(ev[2 * i + 1]);
      if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev[2 * i], ev[2 * i + 1]);
      if (e != hipSuccess) { note_hip_error(e); rc = TRJ_ERR_HIP; }
      sum += ms;
    }
    *h_avg_ms = (float)(sum / pairs);
  }
  for (auto& e : ev) (void)hipEventDestroy(e);
  return rc;
}

int32_t trj_workspace_bytes(const trj_model_desc* desc, int32_t t_max, int32_t b_max,
                            int32_t l_max, size_t* h_bytes) {
  if (!h_bytes) return TRJ_ERR_NULLPTR;
  TRJ_TRY(check_desc(desc));
  if (t_max < 1 || b_max < 1 || l_max < 1) return TRJ_ERR_BAD_SHAPE;
  TuneScope tune_scope;
  Carver c(nullptr);
  StepWs w;
  carve_step(c, *desc, b_max, t_max, l_max, true, &w);
  *h_bytes = align_up(c.off, 256);
  return TRJ_OK;
}

int32_t trj_pack_weight(void* dst, const void* src, int32_t n_out, int32_t n_in, int32_t dtype,
                        int32_t kind, int32_t n_heads, int32_t head_dim, void* stream) {
  if (!dst || !src) return TRJ_ERR_NULLPTR;
  if (dtype != TRJ_F32 && dtype != TRJ_BF16) return TRJ_ERR_BAD_DTYPE;
  if (n_out < 32 || n_in < 16 || (n_out & 31) || (n_in & 15)) return TRJ_ERR_BAD_SHAPE;
  if (kind == TRJ_PACK_QKV) {
    // rows are [q: n_heads*dh | k | v] with k and v of equal size, kv heads dividing n_heads
    const int kv_rows = head_dim > 0 ? n_out - n_heads * head_dim : 0;
    if (n_heads < 1 || head_dim < 32 || (head_dim & 31) || kv_rows < 2 * head_dim ||
        kv_rows % (2 * head_dim) != 0 || n_heads % (kv_rows / (2 * head_dim)) != 0)
      return TRJ_ERR_BAD_SHAPE;
  } else if (kind == TRJ_PACK_GATE_UP) {
    if (n_out & 63) return TRJ_ERR_BAD_SHAPE;
  } else if (kind != TRJ_PACK_PLAIN) {
    return TRJ_ERR_BAD_SHAPE;
  }
  return launch_pack_weight(dst, src, n_out, n_in, dtype, kind, n_heads, head_dim,
                            (hipStream_t)stream);
}

static int kv_convert(void* k_pool, void* v_pool, void* k_plain, void* v_plain, int n_heads,
                      int head_dim, int s_pool, int slot0, int n_slots, int dtype, bool pack,
                      void* stream) {
  if (!k_pool || !v_pool || (n_slots > 0 && (!k_plain || !v_plain))) return TRJ_ERR_NULLPTR;
  if (dtype != TRJ_F32 && dtype != TRJ_BF16) return TRJ_ERR_BAD_DTYPE;
  if (n_heads < 1 || head_dim < 32 || (head_dim & 31) || s_pool < 32 || (s_pool & 31) ||
      slot0 < 0 || n_slots < 0 || (long)slot0 + n_slots > s_pool)
    return TRJ_ERR_BAD_SHAPE;
  return launch_kv_convert(k_pool, v_pool, k_plain, v_plain, n_heads, head_dim, s_pool, slot0,
                           n_slots, dtype, pack, (hipStream_t)stream);
}
int32_t trj_kv_pack(void* k_pool, void* v_pool, const void* k_plain, const void* v_plain,
                    int32_t n_heads, int32_t head_dim, int32_t s_pool, int32_t slot0,
                    int32_t n_slots, int32_t dtype, void* stream) {
  return kv_convert(k_pool, v_pool, const_cast<void*>(k_plain), const_cast<void*>(v_plain),
                    n_heads, head_dim, s_pool, slot0, n_slots, dtype, true, stream);
}
int32_t trj_kv_unpack(void* k_plain, void* v_plain, const void* k_pool, const void* v_pool,
                      int32_t n_heads, int32_t head_dim, int32_t s_pool, int32_t slot0,
                      int32_t n_slots, int32_t dtype, void* stream) {
  return kv_convert(const_cast<void*>(k_pool), const_cast<void*>(v_pool), k_plain, v_plain,
                    n_heads, head_dim, s_pool, slot0, n_slots, dtype, false, stream);
}

// Plain device-to-device copy kernel of a known size: the yardstick against which the
// HBM traffic counters (FETCH_SIZE / WRITE_SIZE) of the other kernels are scaled.
__global__ void copy_probe_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16;
       i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}
int32_t trj_copy_probe(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src) return TRJ_ERR_NULLPTR;
  if (bytes == 0 || (bytes & 15)) return TRJ_ERR_BAD_SHAPE;
  copy_probe_kernel<<<4096, 256, 0, (hipStream_t)stream>>>((const uint4*)src, (uint4*)dst, bytes / 16);
  return check_launch();
}

// Streaming read of a buffer (loads with the streaming hint, nothing stored unless the data
// has one particular value): what a kernel that only reads reaches on this device.
__global__ __launch_bounds__(512) void read_probe_kernel(const u32x4* __restrict__ src, size_t n16,
                                                         uint32_t* __restrict__ sink) {
  u32x4 acc = {0, 0, 0, 0};
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 7 * stride < n16; i += 8 * stride) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u];
  }
  for (; i < n16; i += stride) acc ^= __builtin_nontemporal_load(src + i);
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = 1;
}
int32_t trj_read_probe(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !sink) return TRJ_ERR_NULLPTR;
  if (bytes == 0 || (bytes & 15)) return TRJ_ERR_BAD_SHAPE;
  read_probe_kernel<<<2048, 512, 0, (hipStream_t)stream>>>((const u32x4*)src, bytes / 16, (uint32_t*)sink);
  return check_launch();
}

// What the current device reports about itself (for the peaks a benchmark divides by).
int32_t trj_dev_device_info(int32_t* h_info) {
  if (!h_info) return TRJ_ERR_NULLPTR;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  const hipDeviceAttribute_t attr[6] = {hipDeviceAttributeMultiprocessorCount, hipDeviceAttributeClockRate,
                                        hipDeviceAttributeMemoryClockRate, hipDeviceAttributeMemoryBusWidth,
                                        hipDeviceAttributeL2CacheSize, hipDeviceAttributeMaxSharedMemoryPerBlock};
  for (int i = 0; i < 6 && e == hipSuccess; ++i) {
    int v = 0;
    e = hipDeviceGetAttribute(&v, attr[i], dev);
    h_info[i] = v;
  }
  if (e != hipSuccess) { note_hip_error(e); return TRJ_ERR_HIP; }
  return TRJ_OK;
}

int32_t trj_tree_mask(const int32_t* parent, const int32_t* node_off, int32_t B, int32_t T,
                      int32_t* depth, uint64_t* anc, int32_t* status_dev, void* stream) {
  if (!parent || !node_off || !depth || !anc || !status_dev) return TRJ_ERR_NULLPTR;
  if (B < 1 || T < 1 || T < B) return TRJ_ERR_BAD_SHAPE;
  if ((long)T > (long)B * TRJ_N_MAX) return TRJ_ERR_TREE_TOO_LARGE;
  return launch_tree_prep(parent, node_off, nullptr, nullptr, B, T, 0, 0, depth, anc, status_dev,
                          nullptr, nullptr, nullptr, nullptr, 0, (hipStream_t)stream);
}

// ---- the entry point for callers that cannot allocate: its scratch is this array.
// In host code the array's name is only a stand-in for the symbol; the device address is
// asked for once per device (static_scratch) and that pointer is what kernels receive.
static __device__ __align__(256) unsigned char scratch[TRJ_STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
static void* g_scratch_ptr[MAX_DEVICES];  // per device: each GPU holds its own copy of the array
static std::mutex g_scratch_mu;
static int static_scratch(void** ptr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { trj::note_hip_error(e); return TRJ_ERR_HIP; }
  if (dev < 0 || dev >= MAX_DEVICES) return TRJ_ERR_BAD_SHAPE;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));  // the current device's copy
    if (e != hipSuccess || !p) {
      trj::note_hip_error(e != hipSuccess ? e : hipErrorInvalidSymbol);
      return TRJ_ERR_HIP;
    }
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return TRJ_OK;
}

static int tree_attention_impl(const void* q, const void* k_layer, const void* v_layer,
                       const int32_t* parent, const int32_t* node_off, const int32_t* kv_off,
                       const int32_t* prefix_len, int32_t B, int32_t T, int32_t n_heads,
                       int32_t n_kv_heads, int32_t head_dim, int32_t s_pool, int32_t max_seq_slots,
                       int32_t dtype, float scale, bool static_ws, void* workspace, size_t ws_bytes,
                       void* out, void* stream) {
  if (!q || !k_layer || !v_layer || !parent || !node_off || !kv_off || !prefix_len || !out ||
      (!static_ws && !workspace))
    return TRJ_ERR_NULLPTR;
  if (dtype != TRJ_F32 && dtype != TRJ_BF16) return TRJ_ERR_BAD_DTYPE;
  TRJ_TRY(check_batch(B, T, s_pool, max_seq_slots));
  if (n_heads < 1 || head_dim < 32 || (head_dim & 31)) return TRJ_ERR_BAD_SHAPE;
  if (n_kv_heads == 0) n_kv_heads = n_heads;
  if (n_kv_heads < 1 || n_heads % n_kv_heads != 0) return TRJ_ERR_BAD_SHAPE;
  if (dtype == TRJ_BF16 && head_dim != 64 && head_dim != 128) return TRJ_ERR_BAD_SHAPE;
  if (dtype == TRJ_F32 && (size_t)(head_dim + max_seq_slots) * 4 > 64 * 1024)
    return TRJ_ERR_BAD_SHAPE;
  if (!(scale > 0.f)) return TRJ_ERR_BAD_SHAPE;
  TuneScope tune_scope;
  if (static_ws) {  // sizes first: nothing is touched when the call does not fit the array
    Carver need(nullptr);
    TreeWs wn;
    carve_tree(need, dtype, B, T, n_heads, head_dim, max_seq_slots, &wn);
    if (need.off > (size_t)TRJ_STATIC_SCRATCH_BYTES) return TRJ_ERR_WORKSPACE_TOO_SMALL;
    TRJ_TRY(static_scratch(&workspace));
    ws_bytes = TRJ_STATIC_SCRATCH_BYTES;
  }
  Carver c(workspace);
  TreeWs w;
  carve_tree(c, dtype, B, T, n_heads, head_dim, max_seq_slots, &w);
  if (c.off > ws_bytes) return TRJ_ERR_WORKSPACE_TOO_SMALL;
  hipStream_t st = (hipStream_t)stream;
  TRJ_TRY(launch_tree_prep(parent, node_off, kv_off, prefix_len, B, T, s_pool, max_seq_slots, w.depth,
                           w.anc, w.status, w.row_slot, w.row_pos, w.row_seq,
                           // bf16: rows of malformed sequences read as zeros
                           dtype == TRJ_BF16 ? out : nullptr, (size_t)T * n_heads * head_dim * 2, st));
  if (dtype == TRJ_BF16) {
    TRJ_TRY(launch_attn_items(node_off, prefix_len, kv_off, w.status, B, w.attn_rows, w.attn_qg,
                              w.attn_bpwg, w.attn_ns, w.items, st));
    return launch_tree_attn_bf16((const uint16_t*)q, (const uint16_t*)k_layer,
                                 (const uint16_t*)v_layer, w.anc, node_off, kv_off, prefix_len,
                                 w.status, w.items, B, T, n_heads, n_kv_heads, head_dim, s_pool, max_seq_slots, scale,
                                 w.attn, 0, 0, (uint16_t*)out, st);
  }
  return launch_tree_attn_f32((const float*)q, (const float*)k_layer, (const float*)v_layer, w.anc,
                              w.row_seq, node_off, kv_off, prefix_len, w.status, T, n_heads,
                              n_kv_heads, head_dim, s_pool, max_seq_slots, scale, (float*)out, st);
}

int32_t tree_attention_workspace_bytes(int32_t B, int32_t T, int32_t n_heads, int32_t head_dim,
                                       int32_t max_seq_slots, int32_t dtype, size_t* h_bytes) {
  if (!h_bytes) return TRJ_ERR_NULLPTR;
  if (dtype != TRJ_F32 && dtype != TRJ_BF16) return TRJ_ERR_BAD_DTYPE;
  if (B < 1 || T < B || max_seq_slots < 1 || n_heads < 1 || head_dim < 32 || (head_dim & 31))
    return TRJ_ERR_BAD_SHAPE;
  if ((long)T > (long)B * TRJ_N_MAX) return TRJ_ERR_TREE_TOO_LARGE;
  TuneScope tune_scope;
  Carver c(nullptr);
  TreeWs w;
  carve_tree(c, dtype, B, T, n_heads, head_dim, max_seq_slots, &w);
  *h_bytes = align_up(c.off, 256);
  return TRJ_OK;
}

int32_t tree_attention(const void* q, const void* k_layer, const void* v_layer,
                       const int32_t* parent, const int32_t* node_off, const int32_t* kv_off,
                       const int32_t* prefix_len, int32_t B, int32_t T, int32_t n_heads,
                       int32_t n_kv_heads, int32_t head_dim, int32_t s_pool, int32_t max_seq_slots,
                       int32_t dtype, float scale, void* workspace, size_t ws_bytes, void* out,
                       void* stream) {
  return tree_attention_impl(q, k_layer, v_layer, parent, node_off, kv_off, prefix_len, B, T, n_heads,
                             n_kv_heads, head_dim, s_pool, max_seq_slots, dtype, scale, false,
                             workspace, ws_bytes, out, stream);
}

int32_t tree_attention_static_scratch(const void* q, const void* k_layer, const void* v_layer,
                                      const int32_t* parent, const int32_t* node_off,
                                      const int32_t* kv_off, const int32_t* prefix_len, int32_t B,
                                      int32_t T, int32_t n_heads, int32_t n_kv_heads,
                                      int32_t head_dim, int32_t s_pool, int32_t max_seq_slots,
                                      int32_t dtype, float scale, void* out, void* stream) {
  return tree_attention_impl(q, k_layer, v_layer, parent, node_off, kv_off, prefix_len, B, T, n_heads,
                             n_kv_heads, head_dim, s_pool, max_seq_slots, dtype, scale, true,
                             nullptr, 0, out, stream);
}

int32_t accept_path(const float* logits, const int32_t* tok, const int32_t* parent,
                    const int32_t* node_off, int32_t B, int32_t T, int32_t V, int32_t* argmax_out,
                    int32_t* accept_len, int32_t* best_node, int32_t* path, int32_t* bonus_tok,
                    int32_t* status_dev, void* stream) {
  if (!tok || !parent || !node_off || !argmax_out || !accept_len || !best_node || !path ||
      !bonus_tok || !status_dev)
    return TRJ_ERR_NULLPTR;
  if (B < 1 || T < 1 || T < B || (logits && V < 1)) return TRJ_ERR_BAD_SHAPE;
  if ((long)T > (long)B * TRJ_N_MAX) return TRJ_ERR_TREE_TOO_LARGE;
  hipStream_t st = (hipStream_t)stream;
  if (logits) TRJ_TRY(launch_argmax(logits, T, V, argmax_out, st));
  return launch_accept(argmax_out, tok, parent, node_off, nullptr, B, T, accept_len, best_node,
                       path, bonus_tok, status_dev, st);
}

int32_t kv_compact(void* k_pool, void* v_pool, size_t kv_layer_stride, const int32_t* path,
                   const int32_t* accept_len, const int32_t* kv_off, const int32_t* prefix_len,
                   int32_t B, int32_t n_layers, int32_t n_heads, int32_t head_dim, int32_t s_pool,
                   int32_t dtype, int32_t* new_len, void* stream) {
  if (!k_pool || !v_pool || !path || !accept_len || !kv_off || !prefix_len || !new_len)
    return TRJ_ERR_NULLPTR;
  if (dtype != TRJ_F32 && dtype != TRJ_BF16) return TRJ_ERR_BAD_DTYPE;
  if (B < 1 || n_layers < 1 || n_heads < 1 || head_dim < 32 || (head_dim & 31) || s_pool < 32 ||
      (s_pool & 31) || kv_layer_stride < (size_t)n_heads * s_pool * head_dim)
    return TRJ_ERR_BAD_SHAPE;
  if ((long)n_layers * n_heads > 65535) return TRJ_ERR_BAD_SHAPE;
  return launch_kv_compact(k_pool, v_pool, kv_layer_stride, path, accept_len, kv_off, prefix_len,
                           B, n_layers, n_heads, head_dim, s_pool, dtype, new_len,
                           (hipStream_t)stream);
}

// y[T][n_out] (fp32) = x[T][n_in] * W^T for a TRJ_PACK_PLAIN weight; x plain row-major in
// `dtype`.  Exposes the projection kernel alone (tests, roofline measurements).
// split_k <= 0 picks the library's choice.
int32_t trj_linear(const void* x, const void* w_packed, int32_t T, int32_t n_in, int32_t n_out,
                   int32_t dtype, int32_t split_k, void* workspace, size_t ws_bytes, float* y,
                   void* stream) {
  if (!x || !w_packed || !y || !workspace) return TRJ_ERR_NULLPTR;
  if (dtype != TRJ_F32 && dtype != TRJ_BF16) return TRJ_ERR_BAD_DTYPE;
  if (T < 1 || n_in < 16 || n_out < 32 || (n_in & 15) || (n_out & 31)) return TRJ_ERR_BAD_SHAPE;
  hipStream_t st = (hipStream_t)stream;
  TuneScope tune_scope;
  if (dtype == TRJ_F32)
    return launch_gemm_f32((const float*)x, (const float*)w_packed, T, n_in, n_out, 0, y, st);
  const int tp = padded_rows(T);
  int sk = split_k > 0 ? gemm_bf16_clamp_split(n_out, tp, n_in, split_k) : gemm_bf16_split_k(n_out, tp, n_in);
  Carver c(workspace);
  uint16_t* xp = c.take<uint16_t>((size_t)tp * n_in);
  float* part = c.take<float>((size_t)sk * T * n_out);
  if (c.off > ws_bytes) return TRJ_ERR_WORKSPACE_TOO_SMALL;
  TRJ_TRY(launch_tile_activation((const uint16_t*)x, T, n_in, tp, xp, st));
  const RowScale none{nullptr, 0, tp, 0.f, 0.f};
  if (sk == 1) return launch_gemm_store_f32(xp, (const uint16_t*)w_packed, T, tp, n_in, n_out, 1, none, y, st);
  TRJ_TRY(launch_gemm_store_f32(xp, (const uint16_t*)w_packed, T, tp, n_in, n_out, sk, none, part, st));
  return launch_sum_splits(part, sk, (size_t)T * n_out, y, st);
}

// Which kernel shape a bf16 projection of the step gets: fused != 0 for the QKV and gate/up
// projections (their epilogues rule out a k-split across workgroups), else the split the
// step itself would ask for.
int32_t trj_dev_gemm_plan(int32_t T, int32_t n_in, int32_t n_out, int32_t fused, int32_t* h_plan) {
  if (!h_plan) return TRJ_ERR_NULLPTR;
  if (T < 1 || n_in < 16 || n_out < 32 || (n_in & 15) || (n_out & 31)) return TRJ_ERR_BAD_SHAPE;
  TuneScope tune_scope;
  const int tp = padded_rows(T);
  gemm_bf16_describe_plan(tp, n_in, n_out, fused ? 1 : gemm_bf16_split_k(n_out, tp, n_in), h_plan);
  return TRJ_OK;
}

}  // extern "C"

namespace trj {
// The forward pass over the tree rows; with_head == false stops after the last decoder
// layer (the tree's K/V are in the pool, nothing else is produced), which is what a
// prompt pass needs.
int step_impl(const trj_model_desc* desc, const trj_weights* weights, void* k_pool, void* v_pool,
              size_t kv_layer_stride, int32_t s_pool, const int32_t* tok, const int32_t* parent,
              const int32_t* node_off, const int32_t* kv_off, const int32_t* prefix_len,
              int32_t B, int32_t T, int32_t max_seq_slots, void* workspace, size_t ws_bytes,
              float* logits, int32_t* argmax_out, int32_t* accept_len, int32_t* best_node,
              int32_t* path, int32_t* bonus_tok, int32_t* new_len, int32_t* status_dev,
              bool with_head, hipStream_t st, const TemplateView* tmpl, int max_pos) {
  TRJ_TRY(check_desc(desc));
  if (!weights || !weights->h_layers || !weights->embed || !weights->g_final || !weights->w_lm ||
      !k_pool || !v_pool || !tok || !parent || !node_off || !kv_off || !prefix_len || !workspace ||
      !status_dev)
    return TRJ_ERR_NULLPTR;
  if (with_head &&
      (!argmax_out || !accept_len || !best_node || !path || !bonus_tok || !new_len))
    return TRJ_ERR_NULLPTR;
  const trj_model_desc& m = *desc;
  for (int l = 0; l < m.n_layers; ++l) {
    const trj_layer_weights& lw = weights->h_layers[l];
    if (!lw.g_attn || !lw.wqkv || !lw.wo || !lw.g_ffn || !lw.w_gate_up || !lw.w_down)
      return TRJ_ERR_NULLPTR;
  }
  TRJ_TRY(check_batch(B, T, s_pool, max_seq_slots));
  const int d = m.d_model, H = m.n_heads, dh = m.head_dim, hd = H * dh, F = m.d_ffn, V = m.vocab;
  const int Hkv = m.n_kv_heads ? m.n_kv_heads : H;  // K/V heads (grouped-query attention)
  if (kv_layer_stride < (size_t)Hkv * s_pool * dh || (long)m.n_layers * Hkv > 65535)
    return TRJ_ERR_BAD_SHAPE;
  if (m.dtype == TRJ_F32 && (size_t)(dh + max_seq_slots) * 4 > 64 * 1024) return TRJ_ERR_BAD_SHAPE;

  TuneScope tune_scope;
  Carver c(workspace);
  StepWs w;
  carve_step(c, m, B, T, max_seq_slots, with_head && logits == nullptr, &w);
  if (c.off > ws_bytes) return TRJ_ERR_WORKSPACE_TOO_SMALL;
  float* lg = logits ? logits : w.logits;
  const float scale = 1.0f / sqrtf((float)dh);

  // bf16: the attention output's padding rows and rows of malformed sequences stay zero all step
  const bool bf16 = m.dtype == TRJ_BF16;
  void* zero = bf16 ? w.op : nullptr;
  const size_t zero_bytes = bf16 ? (size_t)padded_rows(T) * hd * 2 : 0;
  // rotary table: one row per tree row, or (with a prepared template) one row per position,
  // found through each row's position
  const float2* cs = w.cs;
  const int32_t* cs_row = nullptr;
  if (tmpl) {
    // what depends on the tree alone comes from the template; one launch does the rest
    TRJ_TRY(launch_template_step_prep(*tmpl, node_off, kv_off, prefix_len, B, T, dh, max_pos, s_pool,
                                      max_seq_slots, status_dev, w.t.row_slot, w.t.row_pos,
                                      w.t.row_seq, w.t.attn_rows, w.t.attn_qg, w.t.attn_bpwg,
                                      w.t.attn_ns, bf16 ? w.t.items : nullptr, zero, zero_bytes, st));
    w.t.depth = tmpl->depth;
    w.t.anc = tmpl->anc;
    cs = tmpl->cs;
    cs_row = w.t.row_pos;
  } else {
    TRJ_TRY(launch_tree_prep(parent, node_off, kv_off, prefix_len, B, T, s_pool, max_seq_slots,
                             w.t.depth, w.t.anc, status_dev, w.t.row_slot, w.t.row_pos, w.t.row_seq,
                             zero, zero_bytes, st));
    TRJ_TRY(launch_rope_table(w.t.row_pos, T, dh, m.rope_theta, w.cs, st));
    if (bf16)
      TRJ_TRY(launch_attn_items(node_off, prefix_len, kv_off, status_dev, B, w.t.attn_rows, w.t.attn_qg,
                                w.t.attn_bpwg, w.t.attn_ns, w.t.items, st));
  }

  if (m.dtype == TRJ_BF16) {
    const int tp = padded_rows(T);
    const int sk_o = gemm_bf16_split_k(d, tp, hd), sk_d = gemm_bf16_split_k(d, tp, F);
    // the norm's division is done by the projection that consumes hp (RowScale)
    const RowScale rs{w.ssq, reduce_norm_parts(d), tp, 1.0f / (float)d, m.rms_eps};
    const RowScale none{nullptr, 0, tp, 0.f, 0.f};
    { ProfScope ps_(KC_REDUCE_NORM, st); TRJ_TRY(launch_embed_norm((const uint16_t*)weights->embed, tok, T, d, V, w.x,
                              weights->h_layers[0].g_attn, tp, w.hp, w.ssq, st)); }
    for (int l = 0; l < m.n_layers; ++l) {
      const trj_layer_weights& lw = weights->h_layers[l];
      uint16_t* kl = (uint16_t*)k_pool + (size_t)l * kv_layer_stride;
      uint16_t* vl = (uint16_t*)v_pool + (size_t)l * kv_layer_stride;
      { ProfScope ps_(KC_GEMM_QKV, st); TRJ_TRY(launch_gemm_qkv(w.hp, (const uint16_t*)lw.wqkv, T, tp, d, H, Hkv, dh, s_pool, rs, cs,
                              cs_row, w.t.row_slot, w.q, kl, vl, st)); }
      TRJ_TRY(launch_tree_attn_bf16(w.q, kl, vl, w.t.anc, node_off, kv_off, prefix_len, status_dev,
                                    w.t.items, B, T, H, Hkv, dh, s_pool, max_seq_slots, scale, w.t.attn, 1, tp,
                                    w.op, st));
      { ProfScope ps_(KC_GEMM_O, st); TRJ_TRY(launch_gemm_store_f32(w.op, (const uint16_t*)lw.wo, T, tp, hd, d, sk_o, none, w.partial, st)); }
      { ProfScope ps_(KC_REDUCE_NORM, st); TRJ_TRY(launch_reduce_norm(w.partial, sk_o, w.x, lw.g_ffn, T, d, tp, w.hp, w.ssq, st)); }
      { ProfScope ps_(KC_GEMM_GATE_UP, st); TRJ_TRY(launch_gemm_gate_up(w.hp, (const uint16_t*)lw.w_gate_up, tp, d, F, rs, w.act, st)); }
      { ProfScope ps_(KC_GEMM_DOWN, st); TRJ_TRY(launch_gemm_store_f32(w.act, (const uint16_t*)lw.w_down, T, tp, F, d, sk_d, none, w.partial, st)); }
      const float* g_next = l + 1 < m.n_layers ? weights->h_layers[l + 1].g_attn : weights->g_final;
      if (!with_head && l + 1 == m.n_layers) break;  // nothing reads the last FFN of a prompt pass
      { ProfScope ps_(KC_REDUCE_NORM, st); TRJ_TRY(launch_reduce_norm(w.partial, sk_d, w.x, g_next, T, d, tp, w.hp, w.ssq, st)); }
    }
    if (!with_head) return TRJ_OK;
    if (!logits) {  // predictions only: argmax in the LM head's epilogue, no logits in memory
      { ProfScope ps_(KC_GEMM_LM, st); TRJ_TRY(launch_gemm_lm_argmax(w.hp, (const uint16_t*)weights->w_lm, T, tp, d, V, rs, w.cand, argmax_out, st)); }
    } else {
      ProfScope ps_(KC_GEMM_LM, st);
      TRJ_TRY(launch_gemm_store_f32(w.hp, (const uint16_t*)weights->w_lm, T, tp, d, V, 1, rs, lg, st));
    }
  } else {
    TRJ_TRY(launch_embed(weights->embed, tok, T, d, V, m.dtype, w.x, st));
    for (int l = 0; l < m.n_layers; ++l) {
      const trj_layer_weights& lw = weights->h_layers[l];
      float* kl = (float*)k_pool + (size_t)l * kv_layer_stride;
      float* vl = (float*)v_pool + (size_t)l * kv_layer_stride;
      TRJ_TRY(launch_rmsnorm_f32(w.x, lw.g_attn, T, d, m.rms_eps, w.h, st));
      TRJ_TRY(launch_gemm_f32(w.h, (const float*)lw.wqkv, T, d, (H + 2 * Hkv) * dh, 0, w.qkv, st));
      TRJ_TRY(launch_rope_kv_f32(w.qkv, cs, cs_row, w.t.row_slot, T, H, Hkv, dh, s_pool, w.qf, kl, vl, st));
      TRJ_TRY(launch_tree_attn_f32(w.qf, kl, vl, w.t.anc, w.t.row_seq, node_off, kv_off, prefix_len,
                                   status_dev, T, H, Hkv, dh, s_pool, max_seq_slots, scale, w.of, st));
      TRJ_TRY(launch_gemm_f32(w.of, (const float*)lw.wo, T, hd, d, 1, w.x, st));
      TRJ_TRY(launch_rmsnorm_f32(w.x, lw.g_ffn, T, d, m.rms_eps, w.h, st));
      TRJ_TRY(launch_gemm_f32(w.h, (const float*)lw.w_gate_up, T, d, 2 * F, 0, w.gu, st));
      TRJ_TRY(launch_silu_mul_f32(w.gu, T, F, w.actf, st));
      TRJ_TRY(launch_gemm_f32(w.actf, (const float*)lw.w_down, T, F, d, 1, w.x, st));
    }
    if (!with_head) return TRJ_OK;
    TRJ_TRY(launch_rmsnorm_f32(w.x, weights->g_final, T, d, m.rms_eps, w.h, st));
    TRJ_TRY(launch_gemm_f32(w.h, (const float*)weights->w_lm, T, d, V, 0, lg, st));
  }
  if (lg) { ProfScope ps_(KC_ARGMAX, st); TRJ_TRY(launch_argmax(lg, T, V, argmax_out, st)); }
  { ProfScope ps_(KC_ACCEPT, st); TRJ_TRY(launch_accept(argmax_out, tok, parent, node_off, status_dev, B, T, accept_len, best_node,
                        path, bonus_tok, status_dev, st)); }
  ProfScope ps_(KC_KV_COMPACT, st);
  return launch_kv_compact(k_pool, v_pool, kv_layer_stride, path, accept_len, kv_off, prefix_len, B,
                           m.n_layers, Hkv, dh, s_pool, m.dtype, new_len, st);
}

// workspace bytes of one step_impl call (pure arithmetic)
size_t step_workspace_bytes(const trj_model_desc& m, int B, int T, int max_seq_slots) {
  TuneScope tune_scope;
  Carver c(nullptr);
  StepWs w;
  carve_step(c, m, B, T, max_seq_slots, true, &w);
  return c.off + 256;
}
int check_model(const trj_model_desc* m) { return check_desc(m); }

// layout of a template buffer; with base == nullptr it only measures
size_t template_carve(void* base, int B, int T, int dh, int max_pos, TemplateView* v) {
  Carver c(base);
  v->hdr = c.take<int32_t>(8);
  v->depth = c.take<int32_t>(T);
  v->anc = c.take<uint64_t>(2 * (size_t)T);
  v->tstatus = c.take<int32_t>(B);
  v->tnoff = c.take<int32_t>((size_t)B + 1);
  v->tseq = c.take<int32_t>(T);
  v->cs = c.take<float2>((size_t)max_pos * (dh / 2));
  return align_up(c.off, 256);
}
static int check_template_args(const trj_model_desc* desc, int B, int T, int max_pos) {
  TRJ_TRY(check_desc(desc));
  if (B < 1 || T < B || max_pos < 1 || max_pos > (1 << 24)) return TRJ_ERR_BAD_SHAPE;
  if ((long)T > (long)B * TRJ_N_MAX) return TRJ_ERR_TREE_TOO_LARGE;
  return TRJ_OK;
}
}  // namespace trj

extern "C" int32_t tr_template_bytes(const trj_model_desc* desc, int32_t B, int32_t T, int32_t max_pos,
                                     size_t* h_bytes) {
  if (!h_bytes) return TRJ_ERR_NULLPTR;
  TRJ_TRY(trj::check_template_args(desc, B, T, max_pos));
  trj::TemplateView v;
  *h_bytes = trj::template_carve(nullptr, B, T, desc->head_dim, max_pos, &v);
  return TRJ_OK;
}

extern "C" int32_t tr_template_prepare(const trj_model_desc* desc, const int32_t* parent,
                                       const int32_t* node_off, int32_t B, int32_t T, int32_t max_pos,
                                       void* tmpl, size_t tmpl_bytes, void* stream) {
  if (!parent || !node_off || !tmpl) return TRJ_ERR_NULLPTR;
  TRJ_TRY(trj::check_template_args(desc, B, T, max_pos));
  trj::TemplateView v;
  if (trj::template_carve(tmpl, B, T, desc->head_dim, max_pos, &v) > tmpl_bytes)
    return TRJ_ERR_WORKSPACE_TOO_SMALL;
  return trj::launch_template_prepare(parent, node_off, B, T, desc->head_dim, max_pos, desc->rope_theta,
                                      v, (hipStream_t)stream);
}

extern "C" int32_t tr_verify_step_template(
    const trj_model_desc* desc, const trj_weights* weights, void* k_pool, void* v_pool,
    size_t kv_layer_stride, int32_t s_pool, const int32_t* tok, const int32_t* parent,
    const int32_t* node_off, const int32_t* kv_off, const int32_t* prefix_len, int32_t B, int32_t T,
    int32_t max_seq_slots, const void* tmpl, size_t tmpl_bytes, int32_t max_pos, void* workspace,
    size_t ws_bytes, float* logits, int32_t* argmax_out, int32_t* accept_len, int32_t* best_node,
    int32_t* path, int32_t* bonus_tok, int32_t* new_len, int32_t* status_dev, void* stream) {
  if (!tmpl) return TRJ_ERR_NULLPTR;
  TRJ_TRY(trj::check_template_args(desc, B, T, max_pos));
  trj::TemplateView v;
  if (trj::template_carve(const_cast<void*>(tmpl), B, T, desc->head_dim, max_pos, &v) > tmpl_bytes)
    return TRJ_ERR_WORKSPACE_TOO_SMALL;
  return trj::step_impl(desc, weights, k_pool, v_pool, kv_layer_stride, s_pool, tok, parent, node_off,
                        kv_off, prefix_len, B, T, max_seq_slots, workspace, ws_bytes, logits,
                        argmax_out, accept_len, best_node, path, bonus_tok, new_len, status_dev,
                        true, (hipStream_t)stream, &v, max_pos);
}

extern "C" int32_t tr_verify_step(const trj_model_desc* desc, const trj_weights* weights, void* k_pool,
                       void* v_pool, size_t kv_layer_stride, int32_t s_pool, const int32_t* tok,
                       const int32_t* parent, const int32_t* node_off, const int32_t* kv_off,
                       const int32_t* prefix_len, int32_t B, int32_t T, int32_t max_seq_slots,
                       void* workspace, size_t ws_bytes, float* logits, int32_t* argmax_out,
                       int32_t* accept_len, int32_t* best_node, int32_t* path, int32_t* bonus_tok,
                       int32_t* new_len, int32_t* status_dev, void* stream) {
  return trj::step_impl(desc, weights, k_pool, v_pool, kv_layer_stride, s_pool, tok, parent, node_off,
                        kv_off, prefix_len, B, T, max_seq_slots, workspace, ws_bytes, logits,
                        argmax_out, accept_len, best_node, path, bonus_tok, new_len, status_dev,
                        true, (hipStream_t)stream);
}
