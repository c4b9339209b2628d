// bf16 projection GEMMs for a small number of token rows (the tree's rows):
//   Y^T[n_out, T] = W[n_out, n_in] * X^T[n_in, T],  fp32 accumulation on the MFMA units.
// With T of 64..128 the product is bound by streaming W once from HBM, so the kernel is
// organised around that stream: W is stored in 32x16 tiles that are exactly one
// v_mfma_f32_32x32x16_bf16 A operand (each lane's 16 bytes, 1 KiB per wavefront load,
// fully coalesced, straight from HBM into registers, no LDS).  The activations (a few
// hundred KiB, L2 resident) are the B operand: they are kept in the same tiled form in
// global memory, staged through LDS once per workgroup and k-chunk, and shared by the
// workgroup's wavefronts.
//
// Workgroup = 4 wavefronts = 2 row tiles (64 output features) x 2 halves of every
// k-chunk; the two k-halves are added through LDS at the end.  grid = (n_out/64,
// split_k, token blocks).  The epilogue functors fuse what follows the projection:
// rotary + KV-cache write (QKV), SiLU(g)*u (gate/up), plain fp32 stores (split-k
// partial sums, logits).
#include "common.h"
#include "kernels.h"

namespace trj {

struct GemmArgs {
  const uint16_t* xp;  // activations, tiled (a_off), tp rows
  const uint16_t* w;   // weights, tiled (w_off)
  int n_in, n_out, tp;
  int chunks_per_split;
};

// acc layout of v_mfma_f32_32x32x16: lane l, register v -> tile row 8*(v/4) + 4*(l/32) +
// v%4, tile column l%32.  Rows are output features, columns are token rows.

// ---- epilogue: fp32 store, y[split][t][n_out]; 4 consecutive features per store
struct EpiStoreF32 {
  float* y;
  int ld, T;
  size_t split_stride;
  __device__ void operator()(const f32x16& acc, int tile, int ttile, int lane, int split) const {
    int t = ttile * 32 + (lane & 31);
    if (t >= T) return;
    float* row = y + split * split_stride + (size_t)t * ld + tile * 32 + 4 * (lane >> 5);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      f32x4 v = {acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]};
      *reinterpret_cast<f32x4*>(row + 8 * g) = v;
    }
  }
};

// ---- epilogue: act = silu(gate) * up, written bf16 in the tiled activation layout.
// A TRJ_PACK_GATE_UP tile holds gate rows 16*tile.. in tile rows 0..15 and the matching
// up rows in tile rows 16..31, i.e. register v pairs with register v + 8.
struct EpiGateUp {
  uint16_t* act;  // tiled, tp rows, d_ffn columns
  int tp;
  __device__ void operator()(const f32x16& acc, int tile, int ttile, int lane, int) const {
    int t = ttile * 32 + (lane & 31);
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      float r[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float gate = acc[4 * g + i], up = acc[8 + 4 * g + i];
        r[i] = gate / (1.0f + __expf(-gate)) * up;
      }
      int f = 16 * tile + 8 * g + 4 * (lane >> 5);
      u32x2 pk = {pack2bf(r[0], r[1]), pack2bf(r[2], r[3])};
      *reinterpret_cast<u32x2*>(act + a_off(t, f, tp)) = pk;
    }
  }
};

// ---- epilogue: rotary on q and k, q stored plain [T][H][dh], k and v into the pool.
struct EpiQKV {
  const float2* cs;         // [T][dh/2] cos, sin of the row's position
  const int32_t* row_slot;  // pool slot of each row, -1 = skip
  uint16_t* q;
  uint16_t* k_layer;
  uint16_t* v_layer;
  int T, n_heads, dh, s_pool;
  __device__ void operator()(const f32x16& acc, int tile, int ttile, int lane, int) const {
    int t = ttile * 32 + (lane & 31);
    if (t >= T) return;
    int slot = row_slot[t];
    if (slot < 0) return;
    const int tph = dh >> 5, hd_tiles = n_heads * tph, half = dh >> 1;
    const int sec = tile / hd_tiles, head = (tile % hd_tiles) / tph, jt = tile % tph;
    const int hh = lane >> 5;
    if (sec < 2) {
      uint16_t* plane = k_layer + (size_t)head * s_pool * dh;
      uint16_t* qrow = q + ((size_t)t * n_heads + head) * dh;
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        int c = 16 * jt + 8 * g + 4 * hh;
        float ra[4], rb[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float2 sc = cs[(size_t)t * half + c + i];
          float a = acc[4 * g + i], b = acc[8 + 4 * g + i];
          ra[i] = a * sc.x - b * sc.y;
          rb[i] = b * sc.x + a * sc.y;
        }
        u32x2 pa = {pack2bf(ra[0], ra[1]), pack2bf(ra[2], ra[3])};
        u32x2 pb = {pack2bf(rb[0], rb[1]), pack2bf(rb[2], rb[3])};
        if (sec == 0) {
          *reinterpret_cast<u32x2*>(qrow + c) = pa;
          *reinterpret_cast<u32x2*>(qrow + c + half) = pb;
        } else {
          *reinterpret_cast<u32x2*>(plane + k_off(slot, c, dh)) = pa;
          *reinterpret_cast<u32x2*>(plane + k_off(slot, c + half, dh)) = pb;
        }
      }
    } else {
      uint16_t* plane = v_layer + (size_t)head * s_pool * dh;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        int c = 32 * jt + 8 * (v >> 2) + 4 * hh + (v & 3);
        plane[v_off(slot, c, dh)] = f2bf(acc[v]);
      }
    }
  }
};

template <int MT, class Epi>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmArgs a, Epi epi) {
  constexpr int CK = MT == 4 ? 8 : 16;  // k-steps (of 16) per chunk
  constexpr int WS = CK / 2;            // k-steps per wavefront and chunk
  constexpr int XL = MT * CK * 64 / 256;  // 16-byte granules of X per thread and chunk
  constexpr int BUF = MT * CK * 64;     // granules per LDS buffer
  extern __shared__ __align__(16) uint8_t smem[];
  u32x4* lds = reinterpret_cast<u32x4*>(smem);

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int rh = wv & 1, kh = wv >> 1;
  const int ntiles = a.n_out >> 5;
  const int tile = blockIdx.x * 2 + rh;
  const bool tile_ok = tile < ntiles;
  const int ksteps = a.n_in >> 4;
  const int nchunks = (ksteps + CK - 1) / CK;
  const int c0 = blockIdx.y * a.chunks_per_split;
  const int c1 = min(nchunks, c0 + a.chunks_per_split);
  const int tb = blockIdx.z, ttiles = a.tp >> 5;
  const u32x4* wp =
      reinterpret_cast<const u32x4*>(a.w) + (size_t)(tile_ok ? tile : 0) * ksteps * 64 + lane;
  const u32x4* xg = reinterpret_cast<const u32x4*>(a.xp);
  const u32x4 zero = {0, 0, 0, 0};

  f32x16 acc[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[m][v] = 0.f;

  u32x4 w0[WS], w1[WS], xr[XL];

  auto load_w = [&](int c, u32x4* dst) {
#pragma unroll
    for (int s = 0; s < WS; ++s) {
      int ks = c * CK + kh * WS + s;
      dst[s] = ks < ksteps ? wp[(size_t)ks * 64] : zero;
    }
  };
  auto load_x = [&](int c) {
#pragma unroll
    for (int it = 0; it < XL; ++it) {
      int g = it * 256 + tid;
      int ksl = g / (MT * 64), rem = g % (MT * 64);
      int ks = c * CK + ksl;
      xr[it] = ks < ksteps ? xg[((size_t)ks * ttiles + tb * MT) * 64 + rem] : zero;
    }
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int it = 0; it < XL; ++it) lds[buf * BUF + it * 256 + tid] = xr[it];
  };
  auto compute = [&](int buf, const u32x4* wr) {
#pragma unroll
    for (int s = 0; s < WS; ++s) {
      int ksl = kh * WS + s;
      bf16x8 wa = __builtin_bit_cast(bf16x8, wr[s]);
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        bf16x8 xb = __builtin_bit_cast(bf16x8, lds[buf * BUF + (ksl * MT + m) * 64 + lane]);
        acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa, xb, acc[m], 0, 0, 0);
      }
    }
  };

  if (c0 < c1) {
    load_w(c0, w0);
    load_x(c0);
    store_x(0);
    __syncthreads();
    for (int c = c0; c < c1; c += 2) {
      // even step: compute buffer 0 / w0, prefetch into buffer 1 / w1
      bool more = c + 1 < c1;
      if (more) { load_w(c + 1, w1); load_x(c + 1); }
      compute(0, w0);
      if (more) store_x(1);
      __syncthreads();
      if (!more) break;
      // odd step
      bool more2 = c + 2 < c1;
      if (more2) { load_w(c + 2, w0); load_x(c + 2); }
      compute(1, w1);
      if (more2) store_x(0);
      __syncthreads();
    }
  }

  // add the two k-halves through LDS (the chunk buffers are free after the last barrier)
  float* red = reinterpret_cast<float*>(smem);
  if (kh == 1) {
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
      for (int v = 0; v < 16; ++v) red[((rh * MT + m) * 16 + v) * 64 + lane] = acc[m][v];
  }
  __syncthreads();
  if (kh == 0 && tile_ok) {
#pragma unroll
    for (int m = 0; m < MT; ++m) {
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[m][v] += red[((rh * MT + m) * 16 + v) * 64 + lane];
      epi(acc[m], tile, tb * MT + m, lane, blockIdx.y);
    }
  }
}

template <class Epi>
static int launch_gemm(const uint16_t* xp, const uint16_t* w, int tp, int n_in, int n_out,
                       int split_k, const Epi& epi, hipStream_t st) {
  int mt = tp == 32 ? 1 : (tp == 64 ? 2 : 4);
  if (tp % (32 * mt) != 0 || (n_in & 15) || (n_out & 31)) return TRJ_ERR_BAD_SHAPE;
  int ck = mt == 4 ? 8 : 16;
  int ksteps = n_in >> 4, nchunks = (ksteps + ck - 1) / ck;
  if (split_k < 1) split_k = 1;
  if (split_k > nchunks) split_k = nchunks;
  int cps = (nchunks + split_k - 1) / split_k;
  GemmArgs a{xp, w, n_in, n_out, tp, cps};
  dim3 grid((n_out / 32 + 1) / 2, split_k, tp / (32 * mt));
  size_t lds = (size_t)2 * mt * ck * 1024;
  if (mt == 1) gemm_bf16_kernel<1, Epi><<<grid, 256, lds, st>>>(a, epi);
  else if (mt == 2) gemm_bf16_kernel<2, Epi><<<grid, 256, lds, st>>>(a, epi);
  else gemm_bf16_kernel<4, Epi><<<grid, 256, lds, st>>>(a, epi);
  return check_launch();
}

// number of grid splits a request for split_k really gets (never an empty split)
int gemm_bf16_clamp_split(int tp, int n_in, int split_k) {
  int mt = tp == 32 ? 1 : (tp == 64 ? 2 : 4);
  int ck = mt == 4 ? 8 : 16;
  int nchunks = ((n_in >> 4) + ck - 1) / ck;
  if (split_k < 1) split_k = 1;
  if (split_k > nchunks) split_k = nchunks;
  int cps = (nchunks + split_k - 1) / split_k;
  return (nchunks + cps - 1) / cps;
}

int gemm_bf16_split_k(int n_out, int tp, int n_in) {
  // enough workgroups for one per compute unit; projections with a fused epilogue
  // never split
  int mt = tp == 32 ? 1 : (tp == 64 ? 2 : 4);
  int ck = mt == 4 ? 8 : 16;
  int groups = ((n_out / 32 + 1) / 2) * (tp / (32 * mt));
  int nchunks = ((n_in >> 4) + ck - 1) / ck;
  int sk = (g_tune.gemm_target_wgs + groups - 1) / groups;
  if (sk > g_tune.max_split_k) sk = g_tune.max_split_k;
  if (sk > nchunks) sk = nchunks;
  if (sk < 1) sk = 1;
  // the number of non-empty splits for the chosen chunks-per-split
  int cps = (nchunks + sk - 1) / sk;
  return (nchunks + cps - 1) / cps;
}

int launch_gemm_store_f32(const uint16_t* xp, const uint16_t* w, int T, int tp, int n_in,
                          int n_out, int split_k, float* y, hipStream_t st) {
  EpiStoreF32 e{y, n_out, T, (size_t)T * n_out};
  return launch_gemm(xp, w, tp, n_in, n_out, split_k, e, st);
}

int launch_gemm_gate_up(const uint16_t* xp, const uint16_t* w, int tp, int n_in, int d_ffn,
                        uint16_t* act, hipStream_t st) {
  EpiGateUp e{act, tp};
  return launch_gemm(xp, w, tp, n_in, 2 * d_ffn, 1, e, st);
}

int launch_gemm_qkv(const uint16_t* xp, const uint16_t* w, int T, int tp, int n_in, int n_heads,
                    int dh, int s_pool, const float2* cs, const int32_t* row_slot, uint16_t* q,
                    uint16_t* k_layer, uint16_t* v_layer, hipStream_t st) {
  EpiQKV e{cs, row_slot, q, k_layer, v_layer, T, n_heads, dh, s_pool};
  return launch_gemm(xp, w, tp, n_in, 3 * n_heads * dh, 1, e, st);
}

// ------------------------------------------------------------------ split-k sum + residual + RMSNorm
// One workgroup per token row: x[t] += sum_s partial[s][t] (fixed order), then
// h = x * g / sqrt(mean(x^2) + eps) written bf16 in the tiled activation layout.  Rows
// t >= T of the padded tile are written as zeros.  n_split == 0: norm only.
constexpr int RN_THREADS = 256, RN_MAXG = 4;
__global__ __launch_bounds__(RN_THREADS) void reduce_norm_kernel(
    const float* __restrict__ partial, int n_split, size_t split_stride, float* __restrict__ x,
    const float* __restrict__ g, int T, int d, int tp, float eps, uint16_t* __restrict__ hp) {
  const int t = blockIdx.x, tid = threadIdx.x;
  const int ngran = d >> 3;
  if (t >= T) {
    const u32x4 z = {0, 0, 0, 0};
    for (int gi = tid; gi < ngran; gi += RN_THREADS)
      *reinterpret_cast<u32x4*>(hp + a_off(t, gi * 8, tp)) = z;
    return;
  }
  float vals[RN_MAXG][8];
  float ss = 0.f;
#pragma unroll
  for (int it = 0; it < RN_MAXG; ++it) {
    int gi = it * RN_THREADS + tid;
    if (gi < ngran) {
      float* xr = x + (size_t)t * d + gi * 8;
      f32x4 a = *reinterpret_cast<f32x4*>(xr), b = *reinterpret_cast<f32x4*>(xr + 4);
      for (int s = 0; s < n_split; ++s) {
        const float* pr = partial + s * split_stride + (size_t)t * d + gi * 8;
        a += *reinterpret_cast<const f32x4*>(pr);
        b += *reinterpret_cast<const f32x4*>(pr + 4);
      }
      if (n_split > 0) {
        *reinterpret_cast<f32x4*>(xr) = a;
        *reinterpret_cast<f32x4*>(xr + 4) = b;
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        vals[it][e] = a[e];
        vals[it][4 + e] = b[e];
        ss += a[e] * a[e] + b[e] * b[e];
      }
    }
  }
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
  __shared__ float part[RN_THREADS / WAVE];
  if ((tid & 63) == 0) part[tid >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int w = 0; w < RN_THREADS / WAVE; ++w) tot += part[w];
  const float inv = 1.0f / sqrtf(tot / d + eps);
#pragma unroll
  for (int it = 0; it < RN_MAXG; ++it) {
    int gi = it * RN_THREADS + tid;
    if (gi < ngran) {
      const float* gg = g + gi * 8;
      u32x4 pk;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        pk[e] = pack2bf(vals[it][2 * e] * gg[2 * e] * inv, vals[it][2 * e + 1] * gg[2 * e + 1] * inv);
      *reinterpret_cast<u32x4*>(hp + a_off(t, gi * 8, tp)) = pk;
    }
  }
}

int launch_reduce_norm(const float* partial, int n_split, float* x, const float* g, int T, int d,
                       int tp, float eps, uint16_t* hp, hipStream_t st) {
  if ((d & 7) || d > 8 * RN_THREADS * RN_MAXG) return TRJ_ERR_BAD_SHAPE;
  reduce_norm_kernel<<<tp, RN_THREADS, 0, st>>>(partial, n_split, (size_t)T * d, x, g, T, d, tp,
                                                eps, hp);
  return check_launch();
}

// y = sum over splits of partial[s] (fixed order); for the stand-alone linear entry point
__global__ void sum_splits_kernel(const float* __restrict__ partial, int n_split, size_t n,
                                  float* __restrict__ y) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float acc = 0.f;
  for (int s = 0; s < n_split; ++s) acc += partial[s * n + i];
  y[i] = acc;
}
int launch_sum_splits(const float* partial, int n_split, size_t n, float* y, hipStream_t st) {
  sum_splits_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(partial, n_split, n, y);
  return check_launch();
}

// plain [T][n] bf16 -> tiled activation layout (zero padded rows); for the stand-alone
// linear entry point
__global__ void tile_activation_kernel(const uint16_t* __restrict__ x, int T, int n, int tp,
                                       uint16_t* __restrict__ xp) {
  const int t = blockIdx.x;
  for (int gi = threadIdx.x; gi < (n >> 3); gi += blockDim.x) {
    u32x4 v = {0, 0, 0, 0};
    if (t < T) v = *reinterpret_cast<const u32x4*>(x + (size_t)t * n + gi * 8);
    *reinterpret_cast<u32x4*>(xp + a_off(t, gi * 8, tp)) = v;
  }
}
int launch_tile_activation(const uint16_t* x, int T, int n, int tp, uint16_t* xp, hipStream_t st) {
  tile_activation_kernel<<<tp, 256, 0, st>>>(x, T, n, tp, xp);
  return check_launch();
}

}  // namespace trj
