// Tree-masked attention, bf16 storage, fp32 softmax and accumulation.
//
// The work is streaming the sequence's K/V once.  A workgroup of 8 wavefronts owns a
// contiguous range of 32-slot blocks of one (sequence, head) and one group of 32 or 64
// query rows (tree nodes); wavefront (kstream, qtile) walks every KS-th block of the range
// for one tile of 32 queries.  K and V blocks are tiled in memory so that each lane's
// 16-byte load is directly an MFMA A operand (1 KiB coalesced per wavefront load, no LDS):
//   S^T[keys, queries] = K[keys, dh] * Q^T          (v_mfma_f32_32x32x16_bf16)
//   O^T[dh, queries]  += V^T[dh, keys] * P^T[keys, queries]
// With keys as the MFMA row dimension each lane holds one query column, so the online
// softmax state (running max, sum, rescale factor) is per lane, and the S^T registers
// are, after conversion to bf16, exactly the B operand of the second product (the V
// tiling stores keys in the order in which S^T leaves them in the registers).
// The ancestor bit rows mask only the blocks that overlap the tree's own slots.
// The next block's K is requested while the current block's P*V runs and its V while
// the next S^T runs, so no second set of registers is needed.
// The wavefronts of a workgroup merge their (m, l, O) through LDS in a fixed tree.  If
// the workgroup covers the whole sequence it writes the normalised rows; otherwise it
// writes an un-normalised partial and a second, small kernel merges the partials of a
// row in split order.  (Merging inside the same launch by "last workgroup to arrive"
// needs device-scope fences; on this multi-die part each of them writes back and
// invalidates a whole L2, which measured 3-4x the cost of the separate launch.)
#include <type_traits>

#include "common.h"
#include "kernels.h"
#include "tree_vis.h"

namespace trj {

constexpr float NEG_BIG = -1e30f;
constexpr int ATTN_WAVES = 8;

struct AttnArgs {
  const uint16_t* q;
  const uint16_t* k_layer;
  const uint16_t* v_layer;
  const uint64_t* anc;
  const int32_t* node_off;
  const int32_t* kv_off;
  const int32_t* prefix_len;
  const int32_t* status_dev;
  int n_heads, group, s_pool, bpwg, nsplit_max, qg_max;  // group = query heads per K/V head
  int n_kv_groups;  // items x K/V heads: sets of workgroups that share K/V blocks
  // work items (sequence, key split, query group) that exist, longest sequence first, and their number
  // (written by the prep kernels): workgroups past the list's end leave at once, and they
  // are the LAST ids of the launch, so the live ones spread evenly over the compute units
  // One record of 8 words per item: sequence, query group, first row, rows, prefix
  // length, first K/V block of the sequence, key split; a workgroup needs nothing else
  // from memory to find its work, and reads record and count together.
  const int32_t* items;
  const int32_t* n_items;
  float scale_log2e;
  // un-normalised partials, one per (sequence, query tile, head, split), stored as the
  // image of the wavefront's accumulator registers: element (mt*16 + v)*64 + lane, so that
  // every store and every load of the merge kernel is a contiguous 256-byte row
  float* po;        // [B*tiles_per_seq][H][nsplit_max][DH/32 * 16 * 64]
  float* pm;        // [B*tiles_per_seq][H][nsplit_max][32] running max (log2 domain)
  float* pl;        // [B*tiles_per_seq][H][nsplit_max][32] sum of weights
  int tiles_per_seq;
  uint16_t* out;
  int tiled, tp;
};


// Online-softmax update of one query tile with one block of 32 keys: S^T accumulators in,
// packed bf16 probabilities out (the B operand of the second product), running max m and
// sum l of this lane's query updated, `alpha` = factor for the O accumulators.
//
// Blocks that lie wholly in the prefix (all but the last few of a sequence) take this
// lean form: no visibility tests; the max works on the raw scores and the scale
// (log2 e / sqrt(dh), > 0) goes into one fused multiply-add per key; v_exp_f32 directly
// (results below the normal range flush to zero, as they should).
__device__ inline void softmax_tile_prefix(const f32x16& sacc, float scale, float& m, float& l,
                                           float& alpha, u32x4 (&pk)[2]) {
  float mx = sacc[0];
#pragma unroll
  for (int v = 1; v < 16; ++v) mx = fmaxf(mx, sacc[v]);
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  const float m_new = fmaxf(m, mx * scale);
  alpha = __builtin_amdgcn_exp2f(m - m_new);
  float lsum = 0.f;
  float p[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    p[v] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[v], scale, -m_new));
    lsum += p[v];
  }
  l = l * alpha + lsum;
  m = m_new;
#pragma unroll
  for (int kg = 0; kg < 2; ++kg)
#pragma unroll
    for (int e = 0; e < 4; ++e) pk[kg][e] = pack2bf(p[8 * kg + 2 * e], p[8 * kg + 2 * e + 1]);
}

// Blocks that overlap the tree's own slots (at most 5 per sequence): ancestor bits decide
// which keys a query sees; a key that is not visible contributes exactly 0, also while
// nothing is visible yet (m == NEG_BIG).
__device__ inline void softmax_tile_tree(const f32x16& sacc, int key0, int hh, int L, uint64_t anc0,
                                         uint64_t anc1, float scale, float& m, float& l,
                                         float& alpha, u32x4 (&pk)[2]) {
  float sv[16];
  float mx = NEG_BIG;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int kk = key0 + 8 * (v >> 2) + 4 * hh + (v & 3);
    const bool vis = tree_key_visible(kk, L, anc0, anc1);
    sv[v] = vis ? sacc[v] * scale : NEG_BIG;
    mx = fmaxf(mx, sv[v]);
  }
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  const float m_new = fmaxf(m, mx);
  alpha = exp2f(m - m_new);
  float lsum = 0.f;
  float p[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    p[v] = sv[v] > -1e29f ? exp2f(sv[v] - m_new) : 0.f;
    lsum += p[v];
  }
  l = l * alpha + lsum;
  m = m_new;
#pragma unroll
  for (int kg = 0; kg < 2; ++kg)
#pragma unroll
    for (int e = 0; e < 4; ++e) pk[kg][e] = pack2bf(p[8 * kg + 2 * e], p[8 * kg + 2 * e + 1]);
}

// O accumulators times alpha; skipped when no query of the wavefront moved its maximum
// (alpha == 1 in every lane), which is the common case once a few blocks have been seen
template <int MTV>
__device__ inline void rescale_o(f32x16 (&o)[MTV], float alpha) {
  if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) == 0) return;
#pragma unroll
  for (int mt = 0; mt < MTV; ++mt)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[mt][v] *= alpha;
}

template <int DH>
__device__ inline void attn_store_row(const AttnArgs& a, int t, int head, int c, u32x2 v) {
  uint16_t* dst = a.tiled ? a.out + a_off(t, head * DH + c, a.tp)
                          : a.out + ((size_t)t * a.n_heads + head) * DH + c;
  *reinterpret_cast<u32x2*>(dst) = v;
}

template <int DH, int NTW, bool XCHG>
__global__ __launch_bounds__(ATTN_WAVES * 64) void tree_attn_bf16_kernel(AttnArgs a) {
  constexpr int KS = ATTN_WAVES / NTW, KSTEPS = DH / 16, MTV = DH / 32;
  constexpr int OW = MTV * 16 * 64;  // floats of one wavefront's O tile
  extern __shared__ __align__(16) float red[];  // NTW * MTV * (KS-1) parts of 1024 floats
  __shared__ float sm_m[ATTN_WAVES][32], sm_l[ATTN_WAVES][32];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nt = wv % NTW, ks = wv / NTW;
  // Workgroup ids go round-robin over the 8 dies (XCDs), each with its own L2.  The
  // workgroups that walk the SAME K/V blocks (with grouped-query attention the query heads
  // of a K/V head) get ids that fall on one die, next to each other in its dispatch order,
  // so that the blocks come from HBM once; the query groups of one (sequence, split) are
  // neighbours in the item list, which puts them n_kv ids apart on the same die whenever
  // the number of K/V heads is a multiple of 8.
  const int slot = blockIdx.x >> 3, kvg = (slot / a.group) * 8 + (blockIdx.x & 7);
  if (kvg >= a.n_kv_groups) return;  // padding to a multiple of 8 (uniform)
  const int n_kv = a.n_heads / a.group;
  const int head = (kvg % n_kv) * a.group + slot % a.group;
  const int item = kvg / n_kv;
  const int32_t* rec = a.items + (size_t)item * 8;  // inside the list's memory for every id
  const int s = rec[0], qg = rec[1], r0 = rec[2], n = rec[3], L = rec[4], blk_base = rec[5];
  const int sp = rec[6];
  if (item >= a.n_items[0]) return;  // uniform over the workgroup, before any barrier
  const int total = L + n;
  const int nb = (total + 31) >> 5;
  const int nsplit = (nb + a.bpwg - 1) / a.bpwg;
  if (sp >= nsplit || qg * 32 * NTW >= n) return;  // uniform as well
  const int b0 = sp * a.bpwg, b1 = min(nb, b0 + a.bpwg);
  const int n32 = lane & 31, hh = lane >> 5;

  // this wavefront's 32 queries: B operands of the first product, kept in registers
  const int qi = (qg * NTW + nt) * 32 + n32;
  const bool valid = qi < n;
  const int qrow = valid ? r0 + qi : -1;
  // rows past the tree's end read the last row instead (never stored, always finite):
  // every load of the prologue is unconditional, so that the query, the ancestor bits and
  // the first K/V block are all in flight together
  const int qc = min(qi, n - 1);
  bf16x8 qreg[KSTEPS];
  {
    const uint16_t* qp = a.q + ((size_t)(r0 + qc) * a.n_heads + head) * DH + hh * 8;
#pragma unroll
    for (int k = 0; k < KSTEPS; ++k)
      qreg[k] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qp + 16 * k));
  }
  uint64_t anc0 = a.anc[2 * (size_t)(r0 + qc)];
  uint64_t anc1 = a.anc[2 * (size_t)(r0 + qc) + 1];

  f32x16 o[MTV];
#pragma unroll
  for (int mt = 0; mt < MTV; ++mt)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[mt][v] = 0.f;
  float m = NEG_BIG, l = 0.f;

  const size_t plane = (size_t)(head / a.group) * a.s_pool * DH;  // the group's K/V head
  const u32x4* kp = reinterpret_cast<const u32x4*>(a.k_layer + plane) + lane;
  const u32x4* vp = reinterpret_cast<const u32x4*>(a.v_layer + plane) + lane;
  u32x4 kreg[KSTEPS], vreg[2 * MTV];  // 1-KiB pieces of a block; V piece mt * 2 + kg
  if (!valid) anc0 = anc1 = 0;        // a row that does not exist sees no tree node

  // The walk over the blocks, compiled once per (HALF, STREAM).
  // NTW == 2: the two wavefronts of a key stream need the same K/V block (one per query
  // tile).  Each loads HALF of its pieces from memory and hands them to the other through
  // LDS (two buffers, one LDS barrier per block; every wavefront makes the same number of
  // trips, one that has run out of blocks reloads its last one and skips the arithmetic),
  // so every byte is asked for once.  (Handing K over before the first product and V
  // before the second, with a barrier each, measured slower at every length.)
  // STREAM: no other workgroup reads these blocks (one query group, one query head per K/V
  // head), so the loads carry the streaming hint; with a second reader shortly after
  // (through L2, or the other wavefront of the pair before the exchange existed) the hint
  // costs a second trip to HBM.
  auto run = [&](auto half_c, auto stream_c) {
    constexpr int HALF = decltype(half_c)::value;
    constexpr bool STREAM = decltype(stream_c)::value;
    constexpr bool PAIR = NTW == 2 && XCHG;
    constexpr int KN = PAIR ? KSTEPS / 2 : KSTEPS, K0 = PAIR ? HALF * KN : 0;
    constexpr int VN = PAIR ? MTV : 2 * MTV, V0 = PAIR ? HALF * VN : 0;
    auto ldg = [&](const u32x4* p) -> u32x4 {
      if constexpr (STREAM) return __builtin_nontemporal_load(p);
      else return *p;
    };
    auto load_k = [&](int blk) {
      const u32x4* kb = kp + (size_t)(blk_base + blk) * KSTEPS * 64;
#pragma unroll
      for (int k = 0; k < KN; ++k) kreg[K0 + k] = ldg(kb + (K0 + k) * 64);
    };
    auto load_v = [&](int blk) {
      const u32x4* vb = vp + (size_t)(blk_base + blk) * MTV * 2 * 64;
#pragma unroll
      for (int i = 0; i < VN; ++i) vreg[V0 + i] = ldg(vb + (V0 + i) * 64);
    };
    u32x4* xch = reinterpret_cast<u32x4*>(red);  // [2 buffers][KS][2 halves][KN + VN][64]
    const int iters = (b1 - b0 + KS - 1) / KS;   // the same for every wavefront
    int b = b0 + ks;
    if (PAIR || b < b1) {
      load_k(min(b, b1 - 1));
      load_v(min(b, b1 - 1));
    }
    for (int it = 0; it < iters; ++it, b += KS) {
      const bool live = b < b1;  // the same for both wavefronts of a stream
      if constexpr (PAIR) {
        constexpr int KO = (HALF ^ 1) * KN, VO = (HALF ^ 1) * VN;
        u32x4* mine = xch + (size_t)((((it & 1) * KS + ks) * 2 + HALF) * (KN + VN)) * 64 + lane;
        const u32x4* theirs =
            xch + (size_t)((((it & 1) * KS + ks) * 2 + (HALF ^ 1)) * (KN + VN)) * 64 + lane;
#pragma unroll
        for (int k = 0; k < KN; ++k) mine[k * 64] = kreg[K0 + k];
#pragma unroll
        for (int i = 0; i < VN; ++i) mine[(KN + i) * 64] = vreg[V0 + i];
        lds_barrier();
#pragma unroll
        for (int k = 0; k < KN; ++k) kreg[KO + k] = theirs[k * 64];
#pragma unroll
        for (int i = 0; i < VN; ++i) vreg[VO + i] = theirs[(KN + i) * 64];
      }
      const bool more = PAIR ? it + 1 < iters : b + KS < b1;
      const int bn = min(b + KS, b1 - 1);
      const int key0 = b * 32;
      f32x16 sacc;
      if (live) {
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[v] = 0.f;
#pragma unroll
        for (int k = 0; k < KSTEPS; ++k)
          sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kreg[k]),
                                                         qreg[k], sacc, 0, 0, 0);
      }
      if (more) load_k(bn);  // uniform branch; in flight during the softmax and P*V
      if (live) {
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
                for (int mt = 0; mt < MTV; ++mt) vreg[mt * 2 + kg][e >> 1] &= keep;
              }
            }
        }
        float alpha;
        u32x4 pk[2];
        if (key0 + 32 > L)
          softmax_tile_tree(sacc, key0, hh, L, anc0, anc1, a.scale_log2e, m, l, alpha, pk);
        else
          softmax_tile_prefix(sacc, a.scale_log2e, m, l, alpha, pk);
        rescale_o<MTV>(o, alpha);
#pragma unroll
        for (int mt = 0; mt < MTV; ++mt)
#pragma unroll
          for (int kg = 0; kg < 2; ++kg)
            o[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                __builtin_bit_cast(bf16x8, vreg[mt * 2 + kg]), __builtin_bit_cast(bf16x8, pk[kg]),
                o[mt], 0, 0, 0);
      }
      if (more) load_v(bn);  // in flight during the next S^T and softmax
    }
  };
  {
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    // uniform over the workgroup; two wavefronts that load the same block rule it out too
    const bool stream = (NTW == 1 || XCHG) && a.group == 1 && rec[7] == 0;
    if (NTW == 2 && XCHG && nt == 1) {
      if (stream) run(I1{}, std::true_type{}); else run(I1{}, std::false_type{});
    } else {
      if (stream) run(I0{}, std::true_type{}); else run(I0{}, std::false_type{});
    }
  }

  // ---- merge the KS key streams of every query tile (fixed order, deterministic)
  const float lt = l + __shfl_xor(l, 32);
  if (hh == 0) {
    sm_m[wv][n32] = m;
    sm_l[wv][n32] = lt;
  }
  __syncthreads();
  float mg = NEG_BIG;
#pragma unroll
  for (int k = 0; k < KS; ++k) mg = fmaxf(mg, sm_m[nt + NTW * k][n32]);
  float lg = 0.f;
#pragma unroll
  for (int k = 0; k < KS; ++k) lg += sm_l[nt + NTW * k][n32] * exp2f(sm_m[nt + NTW * k][n32] - mg);
  {
    const float sc = exp2f(m - mg);
#pragma unroll
    for (int mt = 0; mt < MTV; ++mt)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[mt][v] *= sc;
  }
  // Every key stream keeps the 32-column parts of the output tile it owns (part mt belongs
  // to stream mt % KS) and hands the others over through LDS: one barrier, and the final
  // sums and stores are spread over all wavefronts.  The order of the sum is fixed
  // (own part first, then the other streams in ascending order): deterministic.
  constexpr int PART = 16 * 64;  // floats of one 32-column part of a wavefront's tile
#pragma unroll
  for (int mt = 0; mt < MTV; ++mt) {
    const int owner = mt % KS;
    if (ks != owner) {
      float* dst = red + (((nt * MTV + mt) * (KS - 1)) + (ks < owner ? ks : ks - 1)) * PART + lane;
#pragma unroll
      for (int v = 0; v < 16; ++v) dst[v * 64] = o[mt][v];
    }
  }
  __syncthreads();
  const size_t pidx =
      (((size_t)s * a.tiles_per_seq + qg * NTW + nt) * a.n_heads + head) * a.nsplit_max + sp;
  if (nsplit != 1 && ks == 0 && hh == 0) {
    a.pm[pidx * 32 + n32] = mg;
    a.pl[pidx * 32 + n32] = lg;
  }
  const float inv = 1.0f / lg;
#pragma unroll
  for (int mt = 0; mt < MTV; ++mt) {
    if (ks != mt % KS) continue;
    const float* src = red + ((nt * MTV + mt) * (KS - 1)) * PART + lane;
#pragma unroll
    for (int k = 0; k < KS - 1; ++k)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[mt][v] += src[(k * 16 + v) * 64];
    if (nsplit == 1) {
      // the workgroup saw every key: write the normalised rows
      if (qrow >= 0) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          u32x2 v = {pack2bf(o[mt][4 * g] * inv, o[mt][4 * g + 1] * inv),
                     pack2bf(o[mt][4 * g + 2] * inv, o[mt][4 * g + 3] * inv)};
          attn_store_row<DH>(a, qrow, head, 32 * mt + 8 * g + 4 * hh, v);
        }
      }
    } else {
      // un-normalised partial (merged by attn_combine_kernel): the whole register tile,
      // rows that do not exist included (finite, never read back)
      float* img = a.po + pidx * OW + mt * PART + lane;
#pragma unroll
      for (int v = 0; v < 16; ++v) img[v * 64] = o[mt][v];
    }
  }
}


// Merge the partials of one (sequence, query tile, head) in split order.  512 threads: the
// thread (lane, mt, half) owns the 8 accumulator registers v = 8*half .. 8*half+7 of tile mt
// that lane `lane` of the attention wavefront held, i.e. query lane%32, 8 columns.  The loads
// of a batch of splits are all issued together (clamped, never predicated).
template <int DH>
__global__ __launch_bounds__(512) void attn_combine_kernel(AttnArgs a) {
  constexpr int CB = 8, MTV = DH / 32, OW = MTV * 16 * 64;
  const int tile = blockIdx.x % a.tiles_per_seq, s = blockIdx.x / a.tiles_per_seq;
  const int head = blockIdx.y;
  const int lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const int mt = grp >> 1, v0 = (grp & 1) * 8;
  if (mt >= MTV) return;
  if (a.status_dev[s] != 0) return;  // rows of malformed sequences stay zero
  const int r0 = a.node_off[s], n = a.node_off[s + 1] - r0;
  if (tile * 32 >= n) return;
  const int nb = (a.prefix_len[s] + n + 31) >> 5;
  const int nsplit = (nb + a.bpwg - 1) / a.bpwg;
  if (nsplit == 1) return;  // written by the attention kernel itself
  const int n32 = lane & 31, hh = lane >> 5;
  const size_t base = (((size_t)s * a.tiles_per_seq + tile) * a.n_heads + head) * a.nsplit_max;
  float mrun = NEG_BIG, lrun = 0.f;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int k0 = 0; k0 < nsplit; k0 += CB) {
    float ms[CB], ls[CB], x[CB][8];
#pragma unroll
    for (int j = 0; j < CB; ++j) {
      const int k = min(k0 + j, nsplit - 1);
      ms[j] = a.pm[(base + k) * 32 + n32];
      ls[j] = a.pl[(base + k) * 32 + n32];
      const float* img = a.po + (base + k) * OW + (mt * 16 + v0) * 64 + lane;
#pragma unroll
      for (int e = 0; e < 8; ++e) x[j][e] = img[e * 64];
    }
    float mb = mrun;
#pragma unroll
    for (int j = 0; j < CB; ++j) mb = fmaxf(mb, ms[j]);
    const float resc = exp2f(mrun - mb);
    lrun *= resc;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] *= resc;
#pragma unroll
    for (int j = 0; j < CB; ++j) {
      const float wgt = k0 + j < nsplit ? exp2f(ms[j] - mb) : 0.f;
      lrun += wgt * ls[j];
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += wgt * x[j][e];
    }
    mrun = mb;
  }
  const int qi = tile * 32 + n32;
  if (qi >= n) return;
  const float inv = 1.0f / lrun;
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    u32x2 v = {pack2bf(acc[4 * g] * inv, acc[4 * g + 1] * inv),
               pack2bf(acc[4 * g + 2] * inv, acc[4 * g + 3] * inv)};
    attn_store_row<DH>(a, r0 + qi, head, 32 * mt + 8 * ((v0 >> 2) + g) + 4 * hh, v);
  }
}

// zero fill (rows of malformed sequences and the padding rows of the tiled output)
__global__ void zero_u32_kernel(uint32_t* p, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}
int launch_zero_bytes(void* p, size_t bytes, hipStream_t st) {
  size_t n = bytes / 4;
  if (n == 0) return TRJ_OK;
  zero_u32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>((uint32_t*)p, n);
  return check_launch();
}

// Launch shape: query tiles per workgroup, query groups, blocks per workgroup, splits.
void attn_bf16_plan(int B, int T, int n_heads, int max_seq_slots, int* ntw, int* qg_max, int* bpwg,
                    int* nsplit_max) {
  int nmax = T < TRJ_N_MAX ? T : TRJ_N_MAX;
  *ntw = nmax <= 32 ? 1 : 2;
  *qg_max = (nmax + 32 * *ntw - 1) / (32 * *ntw);
  const int ks = ATTN_WAVES / *ntw;
  int nb = (max_seq_slots + 31) / 32;
  if (nb < 1) nb = 1;
  // the host does not know the trees' sizes (they are device data): the number of work
  // items lies between max(B, T / rows per item) and B * qg_max; the lower figure sizes
  // the split (too few workgroups cost more than too many), the upper one the launch
  const int rows = 32 * *ntw;
  const int items_est = B > (T + rows - 1) / rows ? B : (T + rows - 1) / rows;
  long cols = (long)items_est * n_heads;
  int b = (int)((nb * cols + tune().attn_target_wgs - 1) / tune().attn_target_wgs);
  // shortest walk worth a workgroup, in blocks per wavefront: one for trees of up to 64 nodes
  // (measured at 64 nodes on 1024 slots: 13.7 against 14.1 us; at 16 on 8192: 30 against
  // 32 us), two with two query groups, whose extra workgroups otherwise crowd the launch
  // (128 nodes on 8192 slots: 47.5 against 49 us)
  const int min_bpw = tune().attn_min_bpw > 0 ? tune().attn_min_bpw : (nmax > 64 ? 2 : 1);
  if (b < min_bpw * ks) b = min_bpw * ks;
  if (b > nb) b = nb;
  *bpwg = b;
  *nsplit_max = (nb + b - 1) / b;
}

size_t attn_bf16_ws_floats(int B, int tiles_per_seq, int n_heads, int dh, int nsplit_max) {
  // partials: none needed when every sequence fits one workgroup
  return nsplit_max > 1 ? (size_t)B * tiles_per_seq * n_heads * nsplit_max * (dh / 32 * 1024 + 64)
                        : 64;
}

int launch_tree_attn_bf16(const uint16_t* q, const uint16_t* k_layer, const uint16_t* v_layer,
                          const uint64_t* anc, const int32_t* node_off,
                          const int32_t* kv_off, const int32_t* prefix_len,
                          const int32_t* status_dev, const int32_t* items, int B, int T,
                          int n_heads, int n_kv_heads, int dh, int s_pool, int max_seq_slots,
                          float scale, float* ws, int tiled, int tp, uint16_t* out, hipStream_t st) {
  if (dh != 64 && dh != 128) return TRJ_ERR_BAD_SHAPE;
  int ntw, qg_max, bpwg, nsplit_max;
  attn_bf16_plan(B, T, n_heads, max_seq_slots, &ntw, &qg_max, &bpwg, &nsplit_max);
  const int tiles_per_seq = qg_max * ntw;
  size_t parts = nsplit_max > 1 ? (size_t)B * tiles_per_seq * n_heads * nsplit_max : 0;
  float* po = ws;
  float* pm = ws + parts * (dh / 32 * 1024);
  float* pl = pm + parts * 32;
  AttnArgs a{q, k_layer, v_layer, anc, node_off, kv_off, prefix_len, status_dev, n_heads, n_heads / n_kv_heads,
             s_pool, bpwg, nsplit_max, qg_max, B * qg_max * nsplit_max * n_kv_heads, items,
             items + (size_t)B * qg_max * nsplit_max * 8, scale * 1.4426950408889634f, po, pm, pl, tiles_per_seq, out, tiled, tp};
  const int group = n_heads / n_kv_heads;
  dim3 grid((B * qg_max * n_kv_heads * nsplit_max + 7) / 8 * 8 * group);
  const int ks = ATTN_WAVES / ntw;
  size_t lds = (size_t)ntw * (dh / 32) * (ks - 1) * 16 * 64 * sizeof(float);  // parts handed over
  // With two query tiles per workgroup the wavefront pairs either both load every block, or
  // split the loads and exchange halves through LDS.  The exchange costs a barrier per block
  // and pays once a wavefront walks enough blocks (measured: 2 blocks per wavefront 13.2
  // against 12 us, 8: 33.9 against 31.9, 20: 119 against 137, 32: 89 against 98).
  // It is the streaming hint that pays for it, and the hint needs blocks that nobody else
  // reads: one query head per K/V head, and trees of at most 64 nodes (known here only on
  // average; a sequence with more runs the exchange without the hint, 3-6 % slower than
  // the plain pair).
  const bool xchg = ntw == 2 && bpwg >= tune().attn_xchg_min_blocks && n_heads == n_kv_heads &&
                    T <= 64 * B;
  if (xchg) {  // 2 buffers x streams x halves x pieces
    size_t xch = (size_t)2 * ks * 2 * (dh / 32 + dh / 32) * 1024;
    if (xch > lds) lds = xch;
  }
  {
    ProfScope ps_(KC_ATTN, st);
#define TRJ_ATTN(D, Q, X)                                                                     \
  do {                                                                                        \
    static bool big_lds_allowed = false; /* one-time, per instantiation */                    \
    if (!big_lds_allowed) {                                                                   \
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(tree_attn_bf16_kernel<D, Q, X>), \
                                hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);      \
      big_lds_allowed = true;                                                                 \
    }                                                                                         \
    tree_attn_bf16_kernel<D, Q, X><<<grid, ATTN_WAVES * 64, lds, st>>>(a);                    \
  } while (0)
    if (dh == 128) {
      if (ntw == 1) TRJ_ATTN(128, 1, false); else if (xchg) TRJ_ATTN(128, 2, true); else TRJ_ATTN(128, 2, false);
    } else {
      if (ntw == 1) TRJ_ATTN(64, 1, false); else if (xchg) TRJ_ATTN(64, 2, true); else TRJ_ATTN(64, 2, false);
    }
#undef TRJ_ATTN
  }
  int rc = check_launch();
  if (rc || nsplit_max == 1) return rc;
  ProfScope ps_(KC_ATTN_COMBINE, st);
  dim3 cgrid(B * tiles_per_seq, n_heads);
  if (dh == 128) attn_combine_kernel<128><<<cgrid, 512, 0, st>>>(a);
  else attn_combine_kernel<64><<<cgrid, 512, 0, st>>>(a);
  return check_launch();
}

}  // namespace trj
