// Tree-masked attention, bf16 storage, fp32 softmax and accumulation.
//
// The work is streaming the sequence's K/V once; every wavefront owns a contiguous
// range of 32-slot blocks of one (sequence, head) and up to 64 query rows (tree nodes).
// K and V blocks are tiled in memory so that each lane's 16-byte load is directly an
// MFMA A operand (1 KiB coalesced per wavefront load, no LDS):
//   S^T[keys, queries] = K[keys, dh] * Q^T          (v_mfma_f32_32x32x16_bf16)
//   O^T[dh, queries]  += V^T[dh, keys] * P^T[keys, queries]
// With keys as the MFMA row dimension each lane holds one query column, so the online
// softmax state (running max, sum, rescale factor) is per lane, and the S^T registers
// are, after conversion to bf16, exactly the B operand of the second product (the V
// tiling stores keys in the order in which S^T leaves them in the registers).
// The ancestor bit rows mask only the blocks that overlap the tree's own slots.
// Every wavefront writes an un-normalised partial (m, l, O); a second kernel merges
// the partials of a row in a fixed order.
#include "common.h"
#include "kernels.h"

namespace trj {

struct AttnArgs {
  const uint16_t* q;
  const uint16_t* k_layer;
  const uint16_t* v_layer;
  const uint64_t* anc;
  const int32_t* node_off;
  const int32_t* kv_off;
  const int32_t* prefix_len;
  const int32_t* status_dev;
  int n_heads, s_pool, bpw, nsplit_max, qg_max;
  float scale_log2e;
  float* po;  // [T][H][nsplit_max][DH]
  float* pm;  // [T][H][nsplit_max]
  float* pl;
};

constexpr float NEG_BIG = -1e30f;

template <int DH, int NQT>
__global__ __launch_bounds__(256) void tree_attn_bf16_kernel(AttnArgs a) {
  constexpr int KS = DH / 16, MTV = DH / 32;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int head = blockIdx.y, s = blockIdx.z;
  if (a.status_dev[s] != 0) return;
  const int r0 = a.node_off[s], n = a.node_off[s + 1] - r0;
  const int L = a.prefix_len[s];
  const int total = L + n;
  const int nb = (total + 31) >> 5;
  const int nsplit = (nb + a.bpw - 1) / a.bpw;
  const int wv = blockIdx.x * 4 + w;
  const int qg = wv % a.qg_max, ks = wv / a.qg_max;
  if (ks >= nsplit || qg * 32 * NQT >= n) return;  // whole wavefront leaves; no barriers below
  const int b0 = ks * a.bpw, b1 = min(nb, b0 + a.bpw);
  const int n32 = lane & 31, hh = lane >> 5;

  // queries of this wavefront: B operands of the first product, kept in registers
  bf16x8 qreg[NQT][KS];
  uint64_t anc0[NQT], anc1[NQT];
  int qrow[NQT];
#pragma unroll
  for (int nt = 0; nt < NQT; ++nt) {
    int qi = (qg * NQT + nt) * 32 + n32;
    bool valid = qi < n;
    qrow[nt] = valid ? r0 + qi : -1;
    const uint16_t* qp = a.q + ((size_t)(r0 + (valid ? qi : 0)) * a.n_heads + head) * DH + hh * 8;
#pragma unroll
    for (int k = 0; k < KS; ++k) {
      u32x4 v = {0, 0, 0, 0};
      if (valid) v = *reinterpret_cast<const u32x4*>(qp + 16 * k);
      qreg[nt][k] = __builtin_bit_cast(bf16x8, v);
    }
    anc0[nt] = valid ? a.anc[2 * (size_t)(r0 + qi)] : 0;
    anc1[nt] = valid ? a.anc[2 * (size_t)(r0 + qi) + 1] : 0;
  }

  f32x16 o[NQT][MTV];
  float m[NQT], l[NQT];
#pragma unroll
  for (int nt = 0; nt < NQT; ++nt) {
    m[nt] = NEG_BIG;
    l[nt] = 0.f;
#pragma unroll
    for (int mt = 0; mt < MTV; ++mt)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[nt][mt][v] = 0.f;
  }

  const size_t plane = (size_t)head * a.s_pool * DH;
  const u32x4* kp = reinterpret_cast<const u32x4*>(a.k_layer + plane) + lane;
  const u32x4* vp = reinterpret_cast<const u32x4*>(a.v_layer + plane) + lane;
  const int blk_base = a.kv_off[s] >> 5;

  for (int b = b0; b < b1; ++b) {
    const u32x4* kb = kp + (size_t)(blk_base + b) * KS * 64;
    const u32x4* vb = vp + (size_t)(blk_base + b) * MTV * 2 * 64;
    u32x4 kreg[KS], vreg[MTV][2];
#pragma unroll
    for (int k = 0; k < KS; ++k) kreg[k] = kb[k * 64];
#pragma unroll
    for (int mt = 0; mt < MTV; ++mt)
#pragma unroll
      for (int kg = 0; kg < 2; ++kg) vreg[mt][kg] = vb[(mt * 2 + kg) * 64];

    const int key0 = b * 32;
    const bool need_mask = key0 + 32 > L;
    if (key0 + 32 > total) {
      // slots past the sequence's last row may hold anything (NaN bit patterns too):
      // clear them in the V operand, their probabilities are exactly zero
#pragma unroll
      for (int kg = 0; kg < 2; ++kg)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          int key = key0 + 16 * kg + 4 * hh + 8 * (e >> 2) + (e & 3);
          if (key >= total) {
            uint32_t keep = (e & 1) ? 0x0000ffffu : 0xffff0000u;
#pragma unroll
            for (int mt = 0; mt < MTV; ++mt) vreg[mt][kg][e >> 1] &= keep;
          }
        }
    }

#pragma unroll
    for (int nt = 0; nt < NQT; ++nt) {
      f32x16 sacc;
#pragma unroll
      for (int v = 0; v < 16; ++v) sacc[v] = 0.f;
#pragma unroll
      for (int k = 0; k < KS; ++k)
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kreg[k]),
                                                       qreg[nt][k], sacc, 0, 0, 0);
      float sv[16];
      float mx = NEG_BIG;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        bool vis = true;
        if (need_mask) {
          int kk = key0 + 8 * (v >> 2) + 4 * hh + (v & 3);
          if (kk >= L) {
            int j = kk - L;
            vis = j < 64 ? ((anc0[nt] >> j) & 1) : (j < 128 ? ((anc1[nt] >> (j - 64)) & 1) : 0);
          }
        }
        sv[v] = vis ? sacc[v] * a.scale_log2e : NEG_BIG;
        mx = fmaxf(mx, sv[v]);
      }
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m[nt], mx);
      const float alpha = exp2f(m[nt] - m_new);
      float lsum = 0.f;
      float p[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        p[v] = sv[v] > -1e29f ? exp2f(sv[v] - m_new) : 0.f;
        lsum += p[v];
      }
      l[nt] = l[nt] * alpha + lsum;
      m[nt] = m_new;
      u32x4 pk[2];
#pragma unroll
      for (int kg = 0; kg < 2; ++kg)
#pragma unroll
        for (int e = 0; e < 4; ++e) pk[kg][e] = pack2bf(p[8 * kg + 2 * e], p[8 * kg + 2 * e + 1]);
#pragma unroll
      for (int mt = 0; mt < MTV; ++mt) {
#pragma unroll
        for (int v = 0; v < 16; ++v) o[nt][mt][v] *= alpha;
#pragma unroll
        for (int kg = 0; kg < 2; ++kg)
          o[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              __builtin_bit_cast(bf16x8, vreg[mt][kg]), __builtin_bit_cast(bf16x8, pk[kg]),
              o[nt][mt], 0, 0, 0);
      }
    }
  }

  // partial results of this wavefront
#pragma unroll
  for (int nt = 0; nt < NQT; ++nt) {
    float lt = l[nt] + __shfl_xor(l[nt], 32);
    if (qrow[nt] < 0) continue;
    size_t pidx = ((size_t)qrow[nt] * a.n_heads + head) * a.nsplit_max + ks;
    if (hh == 0) {
      a.pm[pidx] = m[nt];
      a.pl[pidx] = lt;
    }
    float* orow = a.po + pidx * DH;
#pragma unroll
    for (int mt = 0; mt < MTV; ++mt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x4 v = {o[nt][mt][4 * g], o[nt][mt][4 * g + 1], o[nt][mt][4 * g + 2],
                   o[nt][mt][4 * g + 3]};
        *reinterpret_cast<f32x4*>(orow + 32 * mt + 8 * g + 4 * hh) = v;
      }
  }
}

// Merge the partials of every (row, head) in split order; one thread per 8 columns.
// tiled != 0: bf16 output in the tiled activation layout (rows t >= T zero filled),
// else plain [T][H][DH].
template <int DH>
__global__ __launch_bounds__(256) void attn_combine_kernel(
    const float* __restrict__ po, const float* __restrict__ pm, const float* __restrict__ pl,
    const int32_t* __restrict__ row_seq, const int32_t* __restrict__ node_off,
    const int32_t* __restrict__ prefix_len, const int32_t* __restrict__ status_dev, int T,
    int n_heads, int bpw, int nsplit_max, int tiled, int tp, uint16_t* __restrict__ out) {
  const int t = blockIdx.x;
  const int gcol = blockIdx.y * 256 + threadIdx.x;
  const int ncol = n_heads * DH;
  if (gcol * 8 >= ncol) return;
  const int head = gcol * 8 / DH, c = gcol * 8 % DH;
  u32x4 res = {0, 0, 0, 0};
  int s = t < T ? row_seq[t] : -1;
  if (s >= 0 && status_dev[s] == 0) {
    int n = node_off[s + 1] - node_off[s];
    int nb = (prefix_len[s] + n + 31) >> 5;
    int nsplit = (nb + bpw - 1) / bpw;
    size_t base = ((size_t)t * n_heads + head) * nsplit_max;
    float mg = NEG_BIG;
    for (int k = 0; k < nsplit; ++k) mg = fmaxf(mg, pm[base + k]);
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    float lsum = 0.f;
    for (int k = 0; k < nsplit; ++k) {
      float wgt = exp2f(pm[base + k] - mg);
      lsum += wgt * pl[base + k];
      const float* pr = po + (base + k) * DH + c;
      f32x4 x0 = *reinterpret_cast<const f32x4*>(pr), x1 = *reinterpret_cast<const f32x4*>(pr + 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc[e] += wgt * x0[e];
        acc[4 + e] += wgt * x1[e];
      }
    }
    float inv = 1.0f / lsum;
#pragma unroll
    for (int e = 0; e < 4; ++e) res[e] = pack2bf(acc[2 * e] * inv, acc[2 * e + 1] * inv);
  } else if (t < T && !tiled) {
    // rows of malformed sequences: zeros
  }
  if (tiled) {
    *reinterpret_cast<u32x4*>(out + a_off(t, gcol * 8, tp)) = res;
  } else if (t < T) {
    *reinterpret_cast<u32x4*>(out + (size_t)t * ncol + gcol * 8) = res;
  }
}

void attn_bf16_plan(int B, int T, int n_heads, int max_seq_slots, int* nqt, int* qg_max, int* bpw,
                    int* nsplit_max) {
  int nmax = T < TRJ_N_MAX ? T : TRJ_N_MAX;
  *nqt = nmax <= 32 ? 1 : 2;
  *qg_max = (nmax + 32 * *nqt - 1) / (32 * *nqt);
  int nb = (max_seq_slots + 31) / 32;
  if (nb < 1) nb = 1;
  long waves_per_block_col = (long)B * n_heads * *qg_max;
  int b = (int)((nb * waves_per_block_col + g_tune.attn_target_waves - 1) / g_tune.attn_target_waves);
  if (b < g_tune.attn_min_bpw) b = g_tune.attn_min_bpw;
  if (b > nb) b = nb;
  *bpw = b;
  *nsplit_max = (nb + b - 1) / b;
}

size_t attn_bf16_ws_floats(int T, int n_heads, int dh, int nsplit_max) {
  return (size_t)T * n_heads * nsplit_max * (dh + 2);
}

int launch_tree_attn_bf16(const uint16_t* q, const uint16_t* k_layer, const uint16_t* v_layer,
                          const uint64_t* anc, const int32_t* row_seq, const int32_t* node_off,
                          const int32_t* kv_off, const int32_t* prefix_len,
                          const int32_t* status_dev, int B, int T, int n_heads, int dh, int s_pool,
                          int max_seq_slots, float scale, float* ws, int tiled, int tp,
                          uint16_t* out, hipStream_t st) {
  if (dh != 64 && dh != 128) return TRJ_ERR_BAD_SHAPE;
  int nqt, qg_max, bpw, nsplit_max;
  attn_bf16_plan(B, T, n_heads, max_seq_slots, &nqt, &qg_max, &bpw, &nsplit_max);
  size_t rows = (size_t)T * n_heads * nsplit_max;
  float* po = ws;
  float* pm = ws + rows * dh;
  float* pl = pm + rows;
  AttnArgs a{q, k_layer, v_layer, anc, node_off, kv_off, prefix_len, status_dev, n_heads, s_pool,
             bpw, nsplit_max, qg_max, scale * 1.4426950408889634f, po, pm, pl};
  int waves = nsplit_max * qg_max;
  dim3 grid((waves + 3) / 4, n_heads, B);
#define TRJ_ATTN(D, Q) tree_attn_bf16_kernel<D, Q><<<grid, 256, 0, st>>>(a)
  prof_begin(KC_ATTN, st);
  if (dh == 128) { if (nqt == 1) TRJ_ATTN(128, 1); else TRJ_ATTN(128, 2); }
  else { if (nqt == 1) TRJ_ATTN(64, 1); else TRJ_ATTN(64, 2); }
#undef TRJ_ATTN
  prof_end(KC_ATTN, st);
  int rc = check_launch();
  if (rc) return rc;
  int rows_out = tiled ? tp : T;
  dim3 cgrid(rows_out, (n_heads * dh / 8 + 255) / 256);
  ProfScope ps_(KC_ATTN_COMBINE, st);
  if (dh == 128)
    attn_combine_kernel<128><<<cgrid, 256, 0, st>>>(po, pm, pl, row_seq, node_off, prefix_len,
                                                    status_dev, T, n_heads, bpw, nsplit_max, tiled,
                                                    tp, out);
  else
    attn_combine_kernel<64><<<cgrid, 256, 0, st>>>(po, pm, pl, row_seq, node_off, prefix_len,
                                                   status_dev, T, n_heads, bpw, nsplit_max, tiled,
                                                   tp, out);
  return check_launch();
}

}  // namespace trj
