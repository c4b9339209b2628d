// fp32 mode of the verify step: small, plain kernels (fp32 storage, fp32 arithmetic)
// used for the tiny fp32 workload and as a tight-tolerance check of the data layouts.
// They read the same tiled weight / KV layouts as the bf16 kernels.  The element-wise
// kernels at the top (embedding, rotary table) serve both modes.
#include "common.h"
#include "kernels.h"
#include "tree_vis.h"

namespace trj {

// packed row of logical row n (inverse of logical_row)
__device__ inline int packed_row(int n, int kind, int n_out, int n_heads, int dh) {
  if (kind == TRJ_PACK_GATE_UP) {
    int f = n_out >> 1;
    return n < f ? 32 * (n >> 4) + (n & 15) : 32 * ((n - f) >> 4) + 16 + ((n - f) & 15);
  }
  if (kind == TRJ_PACK_QKV) {
    if (n >= n_heads * dh + (n_out - n_heads * dh) / 2) return n;  // v rows
    int base = (n / dh) * dh, c = n % dh, half = dh >> 1;
    return c < half ? base + 32 * (c >> 4) + (c & 15) : base + 32 * ((c - half) >> 4) + 16 + ((c - half) & 15);
  }
  return n;
}

// ------------------------------------------------------------------ rotary table
// cs[t][j] = (cos, sin) of row_pos[t] * theta^(-2j/dh), evaluated in double; without
// row_pos the table is over positions themselves (row t = position t).
__global__ void rope_table_kernel(const int32_t* __restrict__ row_pos, int T, int dh, float theta,
                                  float2* __restrict__ cs) {
  int half = dh >> 1;
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= T * half) return;
  int t = idx / half, j = idx % half;
  double ang = (double)(row_pos ? row_pos[t] : t) * pow((double)theta, -2.0 * j / dh);
  cs[idx] = make_float2((float)cos(ang), (float)sin(ang));
}
int launch_rope_table(const int32_t* row_pos, int T, int dh, float theta, float2* cs,
                      hipStream_t st) {
  int n = T * (dh >> 1);
  rope_table_kernel<<<(n + 255) / 256, 256, 0, st>>>(row_pos, T, dh, theta, cs);
  return check_launch();
}

// ------------------------------------------------------------------ embedding
// x[t][:] = E[tok[t]][:] as fp32.  Token ids outside [0, vocab) are clamped.
template <typename E>
__global__ void embed_kernel(const E* __restrict__ embed, const int32_t* __restrict__ tok, int d,
                             int vocab, float* __restrict__ x) {
  int t = blockIdx.x;
  int id = tok[t];
  id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
  const E* row = embed + (size_t)id * d;
  if constexpr (sizeof(E) == 2) {
    if ((d & 7) == 0) {  // 8 elements per load (rows are 16-byte aligned then)
      const u32x4* r8 = reinterpret_cast<const u32x4*>(row);
      f32x4* x8 = reinterpret_cast<f32x4*>(x + (size_t)t * d);
      for (int g = threadIdx.x; g < (d >> 3); g += blockDim.x) {
        const u32x4 v = r8[g];
        f32x4 lo = {__builtin_bit_cast(float, v.x << 16), __builtin_bit_cast(float, v.x & 0xffff0000u),
                    __builtin_bit_cast(float, v.y << 16), __builtin_bit_cast(float, v.y & 0xffff0000u)};
        f32x4 hi = {__builtin_bit_cast(float, v.z << 16), __builtin_bit_cast(float, v.z & 0xffff0000u),
                    __builtin_bit_cast(float, v.w << 16), __builtin_bit_cast(float, v.w & 0xffff0000u)};
        x8[2 * g] = lo;
        x8[2 * g + 1] = hi;
      }
      return;
    }
  }
  for (int c = threadIdx.x; c < d; c += blockDim.x) {
    if constexpr (sizeof(E) == 2) x[(size_t)t * d + c] = bf2f(row[c]);
    else x[(size_t)t * d + c] = row[c];
  }
}
int launch_embed(const void* embed, const int32_t* tok, int T, int d, int vocab, int dtype,
                 float* x, hipStream_t st) {
  if (dtype == TRJ_BF16)
    embed_kernel<uint16_t><<<T, 512, 0, st>>>((const uint16_t*)embed, tok, d, vocab, x);
  else
    embed_kernel<float><<<T, 256, 0, st>>>((const float*)embed, tok, d, vocab, x);
  return check_launch();
}

// ------------------------------------------------------------------ RMSNorm (fp32 out)
__global__ __launch_bounds__(256) void rmsnorm_f32_kernel(const float* __restrict__ x,
                                                          const float* __restrict__ g, int d,
                                                          float eps, float* __restrict__ h) {
  const float* row = x + (size_t)blockIdx.x * d;
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += 256) ss += row[c] * row[c];
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
  __shared__ float part[4];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = part[0] + part[1] + part[2] + part[3];
  float inv = 1.0f / sqrtf(tot / d + eps);
  for (int c = threadIdx.x; c < d; c += 256) h[(size_t)blockIdx.x * d + c] = row[c] * g[c] * inv;
}
int launch_rmsnorm_f32(const float* x, const float* g, int T, int d, float eps, float* h,
                       hipStream_t st) {
  rmsnorm_f32_kernel<<<T, 256, 0, st>>>(x, g, d, eps, h);
  return check_launch();
}

// ------------------------------------------------------------------ GEMM (fp32)
// y[t][r] (+)= sum_k x[t][k] * W(r, k) for packed rows r.  Block: 32 packed rows x 8
// tokens; consecutive threads read consecutive 32-byte granules of one weight tile.
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ x,
                                                       const float* __restrict__ w, int T,
                                                       int n_in, int n_out, int add_to,
                                                       float* __restrict__ y) {
  const int rl = threadIdx.x & 31, tl = threadIdx.x >> 5;
  const int rt = blockIdx.x, t = blockIdx.y * 8 + tl;
  if (t >= T) return;
  const int ksteps = n_in >> 4;
  const float* xr = x + (size_t)t * n_in;
  float acc = 0.f;
  for (int ks = 0; ks < ksteps; ++ks) {
    const float* tile = w + ((size_t)rt * ksteps + ks) * 512;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const float4* g4 = reinterpret_cast<const float4*>(tile + (h * 32 + rl) * 8);
      float4 a = g4[0], b = g4[1];
      const float* xx = xr + ks * 16 + h * 8;
      acc = fmaf(a.x, xx[0], acc); acc = fmaf(a.y, xx[1], acc);
      acc = fmaf(a.z, xx[2], acc); acc = fmaf(a.w, xx[3], acc);
      acc = fmaf(b.x, xx[4], acc); acc = fmaf(b.y, xx[5], acc);
      acc = fmaf(b.z, xx[6], acc); acc = fmaf(b.w, xx[7], acc);
    }
  }
  size_t o = (size_t)t * n_out + rt * 32 + rl;
  y[o] = add_to ? y[o] + acc : acc;
}
int launch_gemm_f32(const float* x, const float* w, int T, int n_in, int n_out, int add_to,
                    float* y, hipStream_t st) {
  if (T < 1 || n_in < 16 || n_out < 32 || (n_in & 15) || (n_out & 31)) return TRJ_ERR_BAD_SHAPE;
  dim3 grid(n_out / 32, (T + 7) / 8);
  gemm_f32_kernel<<<grid, 256, 0, st>>>(x, w, T, n_in, n_out, add_to, y);
  return check_launch();
}

// ------------------------------------------------------------------ rotary + KV write
// qkv[t][packed rows] -> q[t][head][c] (rotated), K (rotated) and V into the pool at the
// row's slot.  One block per row, one thread per (head, j < dh/2).
__global__ void rope_kv_f32_kernel(const float* __restrict__ qkv, const float2* __restrict__ cs,
                                   const int32_t* __restrict__ cs_row,
                                   const int32_t* __restrict__ row_slot, int n_heads,
                                   int n_kv_heads, int dh, int s_pool, float* __restrict__ q,
                                   float* __restrict__ k_layer, float* __restrict__ v_layer) {
  const int t = blockIdx.x, half = dh >> 1, hd = n_heads * dh, kvd = n_kv_heads * dh;
  const int n_out = hd + 2 * kvd;
  const float* y = qkv + (size_t)t * n_out;
  const int slot = row_slot[t];
  if (slot < 0) return;  // row of a malformed sequence
  const size_t cbase = (size_t)(cs_row ? cs_row[t] : t) * half;  // table row: the row itself or its position
  for (int idx = threadIdx.x; idx < n_heads * half; idx += blockDim.x) {
    int head = idx / half, j = idx % half;
    float2 c = cs[cbase + j];
    int na = head * dh + j, nb = na + half;
    float qa = y[packed_row(na, TRJ_PACK_QKV, n_out, n_heads, dh)];
    float qb = y[packed_row(nb, TRJ_PACK_QKV, n_out, n_heads, dh)];
    float* qo = q + ((size_t)t * n_heads + head) * dh;
    qo[j] = qa * c.x - qb * c.y;
    qo[j + half] = qb * c.x + qa * c.y;
  }
  for (int idx = threadIdx.x; idx < n_kv_heads * half; idx += blockDim.x) {
    int head = idx / half, j = idx % half;
    float2 c = cs[cbase + j];
    int na = head * dh + j, nb = na + half;
    float ka = y[packed_row(hd + na, TRJ_PACK_QKV, n_out, n_heads, dh)];
    float kb = y[packed_row(hd + nb, TRJ_PACK_QKV, n_out, n_heads, dh)];
    float* kp = k_layer + (size_t)head * s_pool * dh;
    float* vp = v_layer + (size_t)head * s_pool * dh;
    kp[k_off(slot, j, dh)] = ka * c.x - kb * c.y;
    kp[k_off(slot, j + half, dh)] = kb * c.x + ka * c.y;
    vp[v_off(slot, j, dh)] = y[hd + kvd + na];
    vp[v_off(slot, j + half, dh)] = y[hd + kvd + nb];
  }
}
int launch_rope_kv_f32(const float* qkv, const float2* cs, const int32_t* cs_row,
                       const int32_t* row_slot, int T,
                       int n_heads, int n_kv_heads, int dh, int s_pool, float* q, float* k_layer,
                       float* v_layer, hipStream_t st) {
  rope_kv_f32_kernel<<<T, 256, 0, st>>>(qkv, cs, cs_row, row_slot, n_heads, n_kv_heads, dh, s_pool, q,
                                        k_layer, v_layer);
  return check_launch();
}

// ------------------------------------------------------------------ SiLU(g) * u
__global__ void silu_mul_f32_kernel(const float* __restrict__ gu, int F, float* __restrict__ act) {
  const int t = blockIdx.x;
  const float* y = gu + (size_t)t * 2 * F;
  for (int f = threadIdx.x; f < F; f += blockDim.x) {
    float g = y[packed_row(f, TRJ_PACK_GATE_UP, 2 * F, 0, 0)];
    float u = y[packed_row(F + f, TRJ_PACK_GATE_UP, 2 * F, 0, 0)];
    act[(size_t)t * F + f] = g / (1.0f + expf(-g)) * u;
  }
}
int launch_silu_mul_f32(const float* gu, int T, int F, float* act, hipStream_t st) {
  silu_mul_f32_kernel<<<T, 256, 0, st>>>(gu, F, act);
  return check_launch();
}

// ------------------------------------------------------------------ tree attention (fp32)
// One wavefront per (row, head).  Scores of all visible slots are kept in LDS
// (max_slots floats), so the sequence length is limited by the LDS size.
__global__ __launch_bounds__(64) void tree_attn_f32_kernel(
    const float* __restrict__ q, const float* __restrict__ k_layer,
    const float* __restrict__ v_layer, const uint64_t* __restrict__ anc,
    const int32_t* __restrict__ row_seq, const int32_t* __restrict__ node_off,
    const int32_t* __restrict__ kv_off, const int32_t* __restrict__ prefix_len,
    const int32_t* __restrict__ status_dev, int n_heads, int group, int dh, int s_pool,
    int max_slots, float scale, float* __restrict__ out) {
  extern __shared__ float lds[];
  float* qs = lds;            // dh
  float* sc = lds + dh;       // max_slots
  const int t = blockIdx.x, head = blockIdx.y, lane = threadIdx.x;
  float* o = out + ((size_t)t * n_heads + head) * dh;
  const int s = row_seq[t];
  const int L = s < 0 ? 0 : prefix_len[s], i = s < 0 ? 0 : t - node_off[s];
  const int base = s < 0 ? 0 : kv_off[s];
  const int nk = L + i + 1;  // ancestors have smaller indices than i
  if (s < 0 || status_dev[s] != 0 || nk > max_slots) {
    for (int c = lane; c < dh; c += 64) o[c] = 0.f;
    return;
  }
  const float* kp = k_layer + (size_t)(head / group) * s_pool * dh;  // the group's K/V head
  const float* vp = v_layer + (size_t)(head / group) * s_pool * dh;
  const float* qr = q + ((size_t)t * n_heads + head) * dh;
  for (int c = lane; c < dh; c += 64) qs[c] = qr[c];
  __syncthreads();
  const uint64_t a0 = anc[2 * (size_t)t], a1 = anc[2 * (size_t)t + 1];
  float mx = -INFINITY;
  for (int kk = lane; kk < nk; kk += 64) {
    const bool vis = tree_key_visible(kk, L, a0, a1);
    float sv = -INFINITY;
    if (vis) {
      float acc = 0.f;
      for (int c = 0; c < dh; ++c) acc = fmaf(qs[c], kp[k_off(base + kk, c, dh)], acc);
      sv = acc * scale;
    }
    sc[kk] = sv;
    mx = fmaxf(mx, sv);
  }
  for (int o2 = 32; o2 > 0; o2 >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o2));
  float sum = 0.f;
  for (int kk = lane; kk < nk; kk += 64) {
    float p = sc[kk] == -INFINITY ? 0.f : expf(sc[kk] - mx);
    sc[kk] = p;
    sum += p;
  }
  for (int o2 = 32; o2 > 0; o2 >>= 1) sum += __shfl_xor(sum, o2);
  __syncthreads();
  const float inv = 1.0f / sum;
  for (int c = lane; c < dh; c += 64) {
    float acc = 0.f;
    for (int kk = 0; kk < nk; ++kk) {
      float p = sc[kk];
      if (p != 0.f) acc = fmaf(p, vp[v_off(base + kk, c, dh)], acc);
    }
    o[c] = acc * inv;
  }
}
int launch_tree_attn_f32(const float* q, const float* k_layer, const float* v_layer,
                         const uint64_t* anc, const int32_t* row_seq, const int32_t* node_off,
                         const int32_t* kv_off, const int32_t* prefix_len,
                         const int32_t* status_dev, int T, int n_heads, int n_kv_heads, int dh,
                         int s_pool, int max_slots, float scale, float* out, hipStream_t st) {
  size_t lds = (size_t)(dh + max_slots) * sizeof(float);
  if (lds > 64 * 1024) return TRJ_ERR_BAD_SHAPE;
  dim3 grid(T, n_heads);
  tree_attn_f32_kernel<<<grid, 64, lds, st>>>(q, k_layer, v_layer, anc, row_seq, node_off,
                                              kv_off, prefix_len, status_dev, n_heads,
                                              n_heads / n_kv_heads, dh, s_pool, max_slots, scale,
                                              out);
  return check_launch();
}

}  // namespace trj
