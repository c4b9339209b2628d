// Shared device/host helpers of the HIP path: data-layout index functions, bf16
// conversion, vector types for the gfx950 MFMA builtins, launch-error bookkeeping.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/trjacobi.h"

namespace trj {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int WAVE = 64;

// ---- bf16 <-> fp32 (round to nearest even; NaN kept quiet)
__host__ __device__ inline uint16_t f2bf(float f) {
  union { float f; uint32_t u; } c;
  c.f = f;
  uint32_t u = c.u;
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__host__ __device__ inline float bf2f(uint16_t b) {
  union { float f; uint32_t u; } c;
  c.u = ((uint32_t)b) << 16;
  return c.f;
}
// two fp32 -> packed bf16 pair (lo in bits 0..15) with the hardware conversion: one
// v_cvt_pk_bf16_f32 on gfx950, round to nearest even, NaN kept quiet
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ inline uint32_t pack2bf(float lo, float hi) {
  f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
// ---- element-offset functions of the tiled layouts (see include/trjacobi.h)
// weight tile layout: packed row r, column k, n_in columns
__host__ __device__ inline size_t w_off(int r, int k, int n_in) {
  return (((size_t)(r >> 5) * (n_in >> 4) + (k >> 4)) * 64 + ((k & 15) >> 3) * 32 + (r & 31)) * 8 +
         (k & 7);
}
// packed activation layout (bf16 GEMM inputs): row t, column k, tp = rows rounded up to 32;
// k-step major so that one k-step of all rows is contiguous
__host__ __device__ inline size_t a_off(int t, int k, int tp) {
  return (((size_t)(k >> 4) * (tp >> 5) + (t >> 5)) * 64 + ((k & 15) >> 3) * 32 + (t & 31)) * 8 +
         (k & 7);
}
// K plane: slot, column c, head_dim dh
__host__ __device__ inline size_t k_off(int slot, int c, int dh) {
  return (((size_t)(slot >> 5) * (dh >> 4) + (c >> 4)) * 64 + ((c & 15) >> 3) * 32 + (slot & 31)) *
             8 + (c & 7);
}
// V plane
__host__ __device__ inline size_t v_off(int slot, int c, int dh) {
  int w = slot & 15;
  return ((((size_t)(slot >> 5) * (dh >> 5) + (c >> 5)) * 2 + ((slot & 31) >> 4)) * 64 +
          ((w >> 2) & 1) * 32 + (c & 31)) * 8 + (w >> 3) * 4 + (w & 3);
}

// logical row of packed row r for the three weight kinds
__host__ __device__ inline int logical_row(int r, int kind, int n_out, int n_heads, int dh) {
  if (kind == TRJ_PACK_GATE_UP) {
    int t = r >> 5, i = r & 31;
    return i < 16 ? 16 * t + i : (n_out >> 1) + 16 * t + (i - 16);
  }
  if (kind == TRJ_PACK_QKV) {
    // rows are [q: n_heads*dh | k: kv_heads*dh | v: kv_heads*dh]; v rows keep their order
    if (r >= n_heads * dh + (n_out - n_heads * dh) / 2) return r;
    int head_base = (r / dh) * dh;
    int j = (r % dh) >> 5, i = r & 31;
    return head_base + (i < 16 ? 16 * j + i : (dh >> 1) + 16 * j + (i - 16));
  }
  return r;
}

// Workgroup barrier that orders LDS traffic only: each wavefront waits for its own LDS
// operations and then joins the barrier, while its outstanding global loads stay in
// flight (the generic barrier would first drain them, which empties a register prefetch
// ring at every k-chunk).
__device__ inline void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// ---- error bookkeeping (defined in api.hip)
void note_hip_error(hipError_t e);
inline int check_launch() {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    note_hip_error(e);
    return TRJ_ERR_HIP;
  }
  return TRJ_OK;
}

inline size_t elem_bytes(int dtype) { return dtype == TRJ_BF16 ? 2 : 4; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace trj
