// bf16 projection GEMMs for a small number of token rows (the tree's rows):
//   Y^T[n_out, T] = W[n_out, n_in] * X^T[n_in, T],  fp32 accumulation on the MFMA units.
// With T of 64..128 the product is bound by streaming W once from HBM, so the kernel is
// organised around that stream: W is stored in 32x16 tiles that are exactly one
// v_mfma_f32_32x32x16_bf16 A operand (each lane's 16 bytes, 1 KiB per wavefront load,
// fully coalesced, straight from HBM into a ring of registers, no LDS).  The activations
// (a few hundred KiB, L2 resident) are the B operand: they are kept in the same tiled form
// in global memory, staged through LDS in phases and shared by the workgroup's wavefronts.
// The epilogue functors fuse what follows the projection: rotary + KV-cache write (QKV),
// SiLU(g)*u (gate/up), plain fp32 stores (split-k partial sums, logits).
//
// What the measurements on gfx950 dictated (each of these cost 20-40 % when violated):
//  - every global load in the main loop is unconditional (indices clamped, never
//    predicated) and wave-uniform values are made visibly uniform (readfirstlane);
//    otherwise the compiler cannot count the loads in flight and waits for all of them;
//  - the barrier between phases orders LDS traffic only, it does not drain global loads;
//  - the activation loads of a phase are issued at the start of the previous phase, so
//    they are older than every W load issued since and waiting for them costs nothing;
//  - a scheduling barrier keeps each W reload next to the step that freed its register.
//
// Packed batches (from 256 token rows) are a different regime: the weights are re-used by
// every block of 128 rows, the product approaches the matrix units' rate, and what binds
// it is LDS bandwidth and where the re-used weight rows come from.  gemm_t_kernel below
// keeps the structure but gives every wavefront two row tiles and places the workgroups
// that share weight rows on one die.
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace trj {

struct GemmArgs {
  const uint16_t* xp;  // activations, tiled (a_off), tp rows
  const uint16_t* w;   // weights, tiled (w_off)
  int n_in, n_out, tp;
  int chunks_per_split;  // phases per k-split
};

// RMSNorm with the division deferred to the consumer: the producer of the activations
// writes bf16(x * g) (not yet divided by the row's norm) and, per row, partial sums of x^2
// over PARTS column parts; a projection of those activations multiplies its accumulators by
// 1 / sqrt(mean(x^2) + eps) of the token row before its epilogue.  (x*g*inv and (x*g)*inv
// round to bf16 with the same relative error; the product with W is linear in inv.)  The
// producer then needs no row-wide reduction and spreads over the whole chip.
// acc layout of v_mfma_f32_32x32x16: lane l, register v -> tile row 8*(v/4) + 4*(l/32) +
// v%4, tile column l%32.  Rows are output features, columns are token rows.

// ---- epilogue: fp32 store, y[split][t][n_out]; 4 consecutive features per store
template <bool SCALED>
struct EpiStoreF32T {
  static constexpr bool kScaled = SCALED;  // are the accumulators divided by the rows' norms first?
  RowScale rs;
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

// ---- epilogue: greedy argmax without logits (Eq. 1's arg max taken where the logits are
// born).  Every wavefront reduces the 32 vocabulary rows of its tile for each of its 32
// token columns and writes one candidate (value, index) per (token, row tile); a second,
// small kernel picks the winner among a token's candidates.  Lowest index wins ties, NaN
// never wins (a candidate that saw nothing keeps index INT32_MAX).
struct ArgmaxCand {
  float v;
  int32_t i;
};
struct EpiArgmax {
  static constexpr bool kScaled = true;
  RowScale rs;
  ArgmaxCand* cand;  // [T][n_tiles]
  int T, n_tiles;
  __device__ void operator()(const f32x16& acc, int tile, int ttile, int lane, int) const {
    float bv = -INFINITY;
    int bi = INT32_MAX;
#pragma unroll
    for (int v = 0; v < 16; ++v) {  // ascending row index within the lane
      const int row = tile * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
      if (acc[v] > bv || (acc[v] == bv && row < bi)) { bv = acc[v]; bi = row; }
    }
    const float ov = __shfl_xor(bv, 32);
    const int oi = __shfl_xor(bi, 32);
    if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    const int t = ttile * 32 + (lane & 31);
    if (lane < 32 && t < T) cand[(size_t)t * n_tiles + tile] = ArgmaxCand{bv, bi};
  }
};

// ---- epilogue: act = silu(gate) * up, written bf16 in the tiled activation layout.
// A TRJ_PACK_GATE_UP tile holds gate rows 16*tile.. in tile rows 0..15 and the matching
// up rows in tile rows 16..31, i.e. register v pairs with register v + 8.
struct EpiGateUp {
  static constexpr bool kScaled = true;
  RowScale rs;
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
  static constexpr bool kScaled = true;
  RowScale rs;
  const float2* cs;         // [.][dh/2] cos, sin: row t of the table, or row cs_row[t] if given
  const int32_t* cs_row;    // optional: the table is indexed by position, this is each row's
  const int32_t* row_slot;  // pool slot of each row, -1 = skip
  uint16_t* q;
  uint16_t* k_layer;
  uint16_t* v_layer;
  int T, n_heads, n_kv_heads, dh, s_pool;
  __device__ void operator()(const f32x16& acc, int tile, int ttile, int lane, int) const {
    int t = ttile * 32 + (lane & 31);
    if (t >= T) return;
    int slot = row_slot[t];
    if (slot < 0) return;
    // row tiles: n_heads*tph of q, then n_kv_heads*tph of k, then as many of v
    const int tph = dh >> 5, q_tiles = n_heads * tph, kv_tiles = n_kv_heads * tph, half = dh >> 1;
    const int sec = tile < q_tiles ? 0 : (tile < q_tiles + kv_tiles ? 1 : 2);
    const int rel = tile - (sec == 0 ? 0 : (sec == 1 ? q_tiles : q_tiles + kv_tiles));
    const int head = rel / tph, jt = rel % tph;
    const int hh = lane >> 5;
    if (sec < 2) {
      const float2* csr = cs + (size_t)(cs_row ? cs_row[t] : t) * half;
      uint16_t* plane = k_layer + (size_t)head * s_pool * dh;
      uint16_t* qrow = q + ((size_t)t * n_heads + head) * dh;
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        int c = 16 * jt + 8 * g + 4 * hh;
        float ra[4], rb[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float2 sc = csr[c + i];
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

// this lane's token row of each of MT token tiles: the partial sums of squares (all parts
// asked for at once, clamped index; parts beyond the last are ignored when they are summed)
template <int MT>
__device__ inline void row_scale_load(const RowScale& rs, int ttile0, int lane, float (&ssq)[MT][RS_MAX_PARTS]) {
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int p = 0; p < RS_MAX_PARTS; ++p) ssq[m][p] = 0.f;
  if (!rs.ssq) return;  // uniform
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    const int t = (ttile0 + m) * 32 + (lane & 31);
#pragma unroll
    for (int p = 0; p < RS_MAX_PARTS; ++p)  // no arithmetic on the loaded value here: it would wait for it
      ssq[m][p] = rs.ssq[(size_t)min(p, rs.parts - 1) * rs.tp + t];
  }
}
__device__ inline float row_scale_factor(const RowScale& rs, const float (&ssq)[RS_MAX_PARTS]) {
  if (!rs.ssq) return 1.0f;
  float s = 0.f;
#pragma unroll
  for (int p = 0; p < RS_MAX_PARTS; ++p) s += p < rs.parts ? ssq[p] : 0.f;  // fixed order
  return 1.0f / sqrtf(s * rs.inv_d + rs.eps);
}
// a scaled copy for the epilogue (the accumulators themselves stay where they are)
__device__ inline f32x16 scaled(const f32x16& acc, float f) {
  f32x16 r;
#pragma unroll
  for (int v = 0; v < 16; ++v) r[v] = acc[v] * f;
  return r;
}

// Main loop.  Workgroup = RT row tiles x KW k-parts wavefronts, no loader.
// The k-range is walked in phases of PH k-steps; the activations of a phase (PH*MT KiB)
// sit in one of two LDS buffers.  Every wavefront
//   - streams its W tiles through a ring of PF registers that runs across phases, and
//   - at the START of a phase issues its share of the loads for the phase after next
//     (kept in registers), and at the END of the phase stores the previous share to the
//     other LDS buffer, followed by one LDS-only barrier.
// Because the activation loads are older than every W load issued during the phase,
// waiting for them at the phase end never stalls the W ring.
template <int MT, int RT, int KW, int PH, int PF, class Epi>
__global__ __launch_bounds__(RT * KW * 64) void gemm_p_kernel(GemmArgs a, Epi epi) {
  constexpr int NWV = RT * KW;
  constexpr int WS = PH / KW;             // k-steps per wavefront and phase
  constexpr int XG = PH * MT * 64;        // 16-byte granules per phase buffer
  constexpr int XL = XG / (NWV * 64);     // activation loads per lane and phase
  // the weight ring holds PF k-steps: a divisor of a phase's WS steps, or RP whole phases
  constexpr int RP = PF > WS ? PF / WS : 1;
  static_assert(PH % KW == 0 && (WS % PF == 0 || PF % WS == 0) && RP <= 4 &&
                    XG % (NWV * 64) == 0, "phase shape");
  extern __shared__ __align__(16) uint8_t smem[];
  u32x4* lds = reinterpret_cast<u32x4*>(smem);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform, and the compiler knows
  const int rt = wv % RT, kw = wv / RT;
  const int ksteps = a.n_in >> 4;
  const int nph = (ksteps + PH - 1) / PH;
  const int ph0 = blockIdx.y * a.chunks_per_split;
  const int ph1 = min(nph, ph0 + a.chunks_per_split);
  const int tb = blockIdx.z, ttiles = a.tp >> 5;
  const int ntiles = a.n_out >> 5;
  const int tile = blockIdx.x * RT + rt;
  const bool tile_ok = tile < ntiles;
  const u32x4 zero = {0, 0, 0, 0};

  f32x16 acc[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[m][v] = 0.f;
  // the token rows' sums of squares are asked for now (oldest loads of the wavefront) and
  // used only after the main loop
  float ssq[Epi::kScaled ? MT : 1][RS_MAX_PARTS];
  if constexpr (Epi::kScaled) row_scale_load<MT>(epi.rs, tb * MT, lane, ssq);

  if (ph0 < ph1) {
    const int n = (ph1 - ph0) * WS;  // k-steps of this wavefront
    const u32x4* wp =
        reinterpret_cast<const u32x4*>(a.w) + (size_t)(tile_ok ? tile : 0) * ksteps * 64 + lane;
    const u32x4* xg = reinterpret_cast<const u32x4*>(a.xp) + (size_t)tb * MT * 64;
    // all indices are clamped, never predicated
    auto w_load = [&](int i) -> u32x4 {
      i = min(i, n - 1);
      int ph = i / WS, s = i - ph * WS;
      int ks = min((ph0 + ph) * PH + kw * WS + s, ksteps - 1);  // X is zero beyond n_in
      // weights are read once per launch: the streaming hint keeps them from displacing
      // the activations in the caches and measurably raises the rate of the stream
      return __builtin_nontemporal_load(wp + (size_t)ks * 64);
    };
    u32x4 xa[XL];
    auto x_load = [&](int ph) {
      ph = min(ph, ph1 - 1);
#pragma unroll
      for (int j = 0; j < XL; ++j) {
        int g = j * (NWV * 64) + tid;
        int ksl = g / (MT * 64), rem = g - ksl * (MT * 64);
        int ks = ph * PH + ksl;
        xa[j] = xg[(size_t)min(ks, ksteps - 1) * ttiles * 64 + rem];
      }
    };
    // k beyond n_in must contribute nothing: zeroed here, at store time, because a select
    // right after the load would make the wavefront wait for it (and for the whole ring)
    auto x_store = [&](int buf, int ph) {
#pragma unroll
      for (int j = 0; j < XL; ++j) {
        int g = j * (NWV * 64) + tid;
        int ks = ph * PH + g / (MT * 64);
        lds[buf * XG + g] = ks < ksteps ? xa[j] : zero;
      }
    };
    u32x4 wr[PF];
    x_load(ph0);
#pragma unroll
    for (int p = 0; p < PF; ++p) wr[p] = w_load(p);
    x_store(0, ph0);
    x_load(ph0 + 1);
    lds_barrier();
    int i = 0;
    // one phase; PAR = its place in the ring's trip when the ring spans several phases
    auto phase = [&](int ph, auto par_c) {
      constexpr int PAR = decltype(par_c)::value;
      const int buf = (ph - ph0) & 1;
#pragma unroll
      for (int q = 0; q < WS; ++q) {
        const int slot = (PAR * WS + q) % PF;  // compile-time after unrolling
        bf16x8 wa = __builtin_bit_cast(bf16x8, wr[slot]);
#pragma unroll
        for (int m = 0; m < MT; ++m) {
          bf16x8 xb = __builtin_bit_cast(
              bf16x8, lds[buf * XG + ((kw * WS + q) * MT + m) * 64 + lane]);
          acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa, xb, acc[m], 0, 0, 0);
        }
        wr[slot] = w_load(i + q + PF);
        __builtin_amdgcn_sched_barrier(0);  // keep each reload next to its step
      }
      i += WS;
      x_store(buf ^ 1, ph + 1);  // activations of the next phase (unused after the last one)
      lds_barrier();
      x_load(ph + 2);
    };
    for (int ph = ph0; ph < ph1; ph += RP) {
      phase(ph, std::integral_constant<int, 0>{});
      if constexpr (RP >= 2) { if (ph + 1 < ph1) phase(ph + 1, std::integral_constant<int, 1>{}); }
      if constexpr (RP >= 4) {
        if (ph + 2 < ph1) phase(ph + 2, std::integral_constant<int, 2>{});
        if (ph + 3 < ph1) phase(ph + 3, std::integral_constant<int, 3>{});
      }
    }
  }

  if (KW > 1) {
    // add the KW partial sums of a row tile through LDS (all phase reads are behind the
    // last barrier)
    float* red = reinterpret_cast<float*>(smem);
    if (ph0 >= ph1) lds_barrier();
    if (kw > 0) {
#pragma unroll
      for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          red[((((kw - 1) * RT + rt) * MT + m) * 16 + v) * 64 + lane] = acc[m][v];
    }
    lds_barrier();
    if (kw == 0) {
#pragma unroll
      for (int q = 1; q < KW; ++q)
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            acc[m][v] += red[((((q - 1) * RT + rt) * MT + m) * 16 + v) * 64 + lane];
    }
  }
  if (kw == 0 && tile_ok) {
#pragma unroll
    for (int m = 0; m < MT; ++m) {
      if constexpr (Epi::kScaled)
        epi(scaled(acc[m], row_scale_factor(epi.rs, ssq[m])), tile, tb * MT + m, lane, blockIdx.y);
      else
        epi(acc[m], tile, tb * MT + m, lane, blockIdx.y);
    }
  }
}

// k-steps per LDS phase of gemm_p_kernel: 8 with one k-part, 16 otherwise.  Short phases
// bring the activations in bursts of 16-32 KiB per workgroup instead of 64, which disturbs
// the weight stream less (one k-part: gate/up 37.9 -> 35.5 us, LM head 49.4 -> 46.8 us with
// 8 k-steps, 37.3 us with 16, 44.6 us with 4 and a ring of only 4; four k-parts: down
// 23.5 -> 21.8 us with 16 k-steps, worse again with 8).  The weight ring stays 8 k-steps
// deep and then spans two or four phases (16 deep: 36.6 us for gate/up).
constexpr int p_phase(int mt, int kw, int rt = 4) { return rt == 3 ? 12 : (kw == 1 ? 8 : 16); }

template <int MT, int RT, int KW, class Epi>
static void launch_p(const uint16_t* xp, const uint16_t* w, int tp, int n_in, int n_out,
                     int split_k, const Epi& epi, hipStream_t st) {
  constexpr int PH = p_phase(MT, KW, RT);
  constexpr int WS = PH / KW;
  constexpr int PF = WS == 6 ? 6 : (WS < 8 ? 8 : (WS < 16 ? WS : 16));
  int ksteps = n_in >> 4, nph = (ksteps + PH - 1) / PH;
  if (split_k < 1) split_k = 1;
  if (split_k > nph) split_k = nph;
  int pps = (nph + split_k - 1) / split_k;
  split_k = (nph + pps - 1) / pps;
  GemmArgs a{xp, w, n_in, n_out, tp, pps};
  dim3 grid((n_out / 32 + RT - 1) / RT, split_k, tp / (32 * MT));
  size_t lds_x = (size_t)2 * PH * MT * 1024, lds_r = (size_t)(KW - 1) * RT * MT * 4096;
  size_t lds = lds_x > lds_r ? lds_x : lds_r;
  auto kern = gemm_p_kernel<MT, RT, KW, PH, PF, Epi>;
  static bool big_lds_allowed = false;  // one-time, per instantiation
  if (!big_lds_allowed) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    big_lds_allowed = true;
  }
  kern<<<grid, RT * KW * 64, lds, st>>>(a, epi);
}

// Many token rows (packed batches): the same structure with KW = 1, but every wavefront
// owns WT row tiles, so that the MT activation operands it reads from LDS per k-step feed
// WT * MT matrix instructions.  With one row tile per wavefront a k-step reads 4 KiB of
// LDS per 4 instructions, which saturates the LDS (128 B/clk per CU) at about a quarter of
// the matrix peak; two row tiles halve that.
template <int MT, int RT, int WT, int PH, int PF, class Epi>
__global__ __launch_bounds__(RT * 64) void gemm_t_kernel(GemmArgs a, Epi epi) {
  constexpr int XG = PH * MT * 64;   // 16-byte granules per phase buffer
  constexpr int XL = XG / (RT * 64);  // activation loads per lane and phase
  static_assert(PH % PF == 0 && XG % (RT * 64) == 0, "phase shape");
  extern __shared__ __align__(16) uint8_t smem[];
  u32x4* lds = reinterpret_cast<u32x4*>(smem);

  const int tid = threadIdx.x, lane = tid & 63;
  const int rt = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ksteps = a.n_in >> 4;
  const int nph = (ksteps + PH - 1) / PH;
  const int ph0 = blockIdx.y * a.chunks_per_split;
  const int ph1 = min(nph, ph0 + a.chunks_per_split);
  // Workgroup ids go round-robin over the 8 dies (XCDs), each with its own L2.  The
  // workgroups that stream the SAME weight rows (one per block of token rows) are given
  // ids that land on one die, next to each other in its dispatch order, so that the rows
  // come from HBM once and are shared through that die's L2; spread over the dies, or far
  // apart in time, every token block re-streams them from HBM.
  const int ttiles = a.tp >> 5, tblocks = ttiles / MT;
  const int ntiles = a.n_out >> 5;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int tb = slot % tblocks, rg = (slot / tblocks) * 8 + xcd;
  if (rg * RT * WT >= ntiles) return;  // padding of the row groups to a multiple of 8 (uniform)
  const int tile0 = (rg * RT + rt) * WT;
  const u32x4 zero = {0, 0, 0, 0};

  f32x16 acc[WT][MT];
#pragma unroll
  for (int r = 0; r < WT; ++r)
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[r][m][v] = 0.f;

  if (ph0 < ph1) {
    const int n = (ph1 - ph0) * PH;  // k-steps of this wavefront
    const u32x4* wp[WT];
#pragma unroll
    for (int r = 0; r < WT; ++r)
      wp[r] = reinterpret_cast<const u32x4*>(a.w) + (size_t)min(tile0 + r, ntiles - 1) * ksteps * 64 + lane;
    const u32x4* xg = reinterpret_cast<const u32x4*>(a.xp) + (size_t)tb * MT * 64;
    // all indices are clamped, never predicated
    auto w_load = [&](int i, int r) -> u32x4 {
      int ks = min(ph0 * PH + min(i, n - 1), ksteps - 1);  // X is zero beyond n_in
      return wp[r][(size_t)ks * 64];
    };
    u32x4 xa[XL];
    auto x_load = [&](int ph) {
      ph = min(ph, ph1 - 1);
#pragma unroll
      for (int j = 0; j < XL; ++j) {
        int g = j * (RT * 64) + tid;
        int ksl = g / (MT * 64), rem = g - ksl * (MT * 64);
        xa[j] = xg[(size_t)min(ph * PH + ksl, ksteps - 1) * ttiles * 64 + rem];
      }
    };
    auto x_store = [&](int buf, int ph) {
#pragma unroll
      for (int j = 0; j < XL; ++j) {
        int g = j * (RT * 64) + tid;
        int ks = ph * PH + g / (MT * 64);
        lds[buf * XG + g] = ks < ksteps ? xa[j] : zero;
      }
    };
    u32x4 wr[PF][WT];
    x_load(ph0);
#pragma unroll
    for (int p = 0; p < PF; ++p)
#pragma unroll
      for (int r = 0; r < WT; ++r) wr[p][r] = w_load(p, r);
    x_store(0, ph0);
    x_load(ph0 + 1);
    lds_barrier();
    int i = 0;
    u32x4 xb[2][MT];  // B operands of the current and the next k-step (LDS latency hidden)
    for (int ph = ph0; ph < ph1; ++ph) {
      const int buf = (ph - ph0) & 1;
      const u32x4* xl = lds + buf * XG + lane;
#pragma unroll
      for (int m = 0; m < MT; ++m) xb[0][m] = xl[m * 64];
#pragma unroll
      for (int q = 0; q < PH; ++q) {
        const int p = q % PF;
        if (q + 1 < PH) {  // compile-time: request the next step's operands first
#pragma unroll
          for (int m = 0; m < MT; ++m) xb[(q + 1) & 1][m] = xl[((q + 1) * MT + m) * 64];
        }
#pragma unroll
        for (int r = 0; r < WT; ++r) {
          bf16x8 wa = __builtin_bit_cast(bf16x8, wr[p][r]);
#pragma unroll
          for (int m = 0; m < MT; ++m)
            acc[r][m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                wa, __builtin_bit_cast(bf16x8, xb[q & 1][m]), acc[r][m], 0, 0, 0);
          wr[p][r] = w_load(i + q + PF, r);
        }
        __builtin_amdgcn_sched_barrier(0);  // keep each reload next to its step
      }
      i += PH;
      x_store(buf ^ 1, ph + 1);  // activations of the next phase (unused after the last one)
      lds_barrier();
      x_load(ph + 2);
    }
  }
  // the rows' norms are fetched only now: this kernel runs for a long time and has no
  // registers to spare for them during the main loop
  float rsf[MT];
  if constexpr (Epi::kScaled) {
    float ssq[MT][RS_MAX_PARTS];
    row_scale_load<MT>(epi.rs, tb * MT, lane, ssq);
#pragma unroll
    for (int m = 0; m < MT; ++m) rsf[m] = row_scale_factor(epi.rs, ssq[m]);
  }
#pragma unroll
  for (int r = 0; r < WT; ++r)
    if (tile0 + r < ntiles) {
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        if constexpr (Epi::kScaled) epi(scaled(acc[r][m], rsf[m]), tile0 + r, tb * MT + m, lane, blockIdx.y);
        else epi(acc[r][m], tile0 + r, tb * MT + m, lane, blockIdx.y);
      }
    }
}

constexpr int BIG_PH = 8, BIG_PF = 4;  // phase and ring of the many-rows kernel
template <int MT, int RT, int WT, class Epi>
static void launch_t(const uint16_t* xp, const uint16_t* w, int tp, int n_in, int n_out,
                     int split_k, const Epi& epi, hipStream_t st) {
  constexpr int PH = BIG_PH, PF = BIG_PF;
  int ksteps = n_in >> 4, nph = (ksteps + PH - 1) / PH;
  if (split_k < 1) split_k = 1;
  if (split_k > nph) split_k = nph;
  int pps = (nph + split_k - 1) / split_k;
  split_k = (nph + pps - 1) / pps;
  GemmArgs a{xp, w, n_in, n_out, tp, pps};
  const int rowgroups = (n_out / 32 + RT * WT - 1) / (RT * WT), tblocks = tp / (32 * MT);
  dim3 grid((rowgroups + 7) / 8 * 8 * tblocks, split_k, 1);
  size_t lds = (size_t)2 * PH * MT * 1024;
  auto kern = gemm_t_kernel<MT, RT, WT, PH, PF, Epi>;
  static bool big_lds_allowed = false;  // one-time, per instantiation
  if (!big_lds_allowed) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    big_lds_allowed = true;
  }
  kern<<<grid, RT * 64, lds, st>>>(a, epi);
}

// (RT, KW) per shape: enough workgroups to cover the chip and enough wavefronts in flight
// (about 700 x 16 KiB saturate HBM here), with as many rows per workgroup as that allows,
// because a workgroup re-reads the whole activation slice for its rows.
struct GemmPlan {
  int mt, rt, kw, wt, ph, split_k;
  bool big;
};
static GemmPlan plan_gemm(int tp, int n_in, int n_out, int split_k) {
  GemmPlan g;
  g.mt = tp <= 96 ? tp / 32 : 4;
  const int ntiles = n_out >> 5, tblocks = tp / (32 * g.mt);
  if (split_k < 1) split_k = 1;
  auto splits = [&](int ph) {  // grid splits a request really gets: never an empty one
    int nph = ((n_in >> 4) + ph - 1) / ph;
    int sk = split_k > nph ? nph : split_k;
    int pps = (nph + sk - 1) / sk;
    return (nph + pps - 1) / pps;
  };
  // many token rows: wavefronts that own two row tiles (see gemm_t_kernel), if that still
  // gives the launch enough workgroups
  // many-rows kernel: 2 or 4 row tiles per wavefront.  Four halve the LDS reads per matrix
  // instruction but leave one workgroup per compute unit, so they pay off only when the
  // launch's last round of 256 workgroups is well filled (measured at 1024 token rows:
  // faster by 5-10 % for 12288, 16384, 28672, 32000, 65536 output rows, slower by 10 % for
  // 22016, where the last round is a third full); split-k launches stay with two.
  g.wt = 2;
  if (tune().gemm_big_wt == 4) g.wt = 4;
  else if (tune().gemm_big_wt == 0 && split_k == 1) {
    const long wgs4 = (long)((ntiles + 15) / 16) * tblocks;
    const long last = wgs4 % 256;
    if (wgs4 >= 128 && (last == 0 || last >= 154)) g.wt = 4;
  }
  const int rgt = 4 * g.wt;  // row tiles per workgroup of the many-rows kernel
  g.big = g.mt == 4 && tune().gemm_big_t > 0 && tp >= tune().gemm_big_t &&
          (long)((ntiles + rgt - 1) / rgt) * tblocks * splits(BIG_PH) >= 128;
  g.ph = g.big ? BIG_PH : (g.mt >= 3 ? 16 : 32);  // provisional: the shape decides it below
  g.split_k = splits(g.ph);
  int shape = tune().gemm_cfg;  // 0 = choose; 1 = (4,1), 2 = (2,4), 3 = (2,2), 4 = (4,2), 5 = (1,8), 6 = (3,2)
  if (shape == 0) shape = (long)ntiles * g.split_k * tblocks >= 4 * 160 ? 1 : 3;
  // 128 token rows: twice the MFMA work per weight byte; two k-parts per row tile keep
  // more wavefronts on the stream (gate/up 58.7 -> 51.1 us)
  if (shape == 1 && g.mt >= 3 && tune().gemm_cfg == 0) shape = 4;
  // What a launch of this kind is bound by is the rate at which ONE compute unit pulls its
  // bytes (weights of its rows plus all activations of its k-range, about 46 GB/s each), so
  // row tiles are spread over as many compute units as there are: when four tiles per
  // workgroup leave a quarter of them idle and three do not overfill them, three tiles and
  // two k-parts (gate/up at 64 rows: 172 -> 230 workgroups, 35.7 -> 34.1 us)
  if (shape == 1 && tune().gemm_cfg == 0 && g.split_k == 1 && tblocks == 1 && (ntiles + 3) / 4 <= 192 &&
      (ntiles + 2) / 3 <= 256)
    shape = 6;
  // long k-range per workgroup: four k-parts (8 wavefronts) keep twice the loads in flight
  // per compute unit (128 rows: QKV 41.1 -> 35.2 us, down 33.2 -> 31.3 us); the output
  // projection's 64 k-steps per split are too short for it (128 rows: 17.3 against 18.0 us;
  // 64 rows: 12.9 against 13.7 us)
  if (shape == 3 && tune().gemm_cfg == 0 && (n_in >> 4) / g.split_k >= 128) shape = 2;
  // few row tiles (the QKV projection of a grouped-query model: 192): one row tile per
  // workgroup and eight k-parts, so that the launch still has a workgroup on most compute
  // units (one compute unit pulls at most ~48 GB/s): 22.8 -> 20.2 us for 6144 x 4096
  if (shape == 2 && tune().gemm_cfg == 0 && (long)ntiles * g.split_k * tblocks <= 256) shape = 5;
  g.rt = (shape == 1 || shape == 4) ? 4 : (shape == 5 ? 1 : (shape == 6 ? 3 : 2));
  g.kw = shape == 1 ? 1 : (shape == 2 ? 4 : (shape == 5 ? 8 : 2));
  if (g.big) { g.rt = 4; g.kw = 1; }
  else {
    g.ph = p_phase(g.mt, g.kw, g.rt);
    g.split_k = splits(g.ph);  // what launch_p computes from the same request
  }
  return g;
}

template <class Epi>
static int launch_gemm(const uint16_t* xp, const uint16_t* w, int tp, int n_in, int n_out,
                       int split_k, const Epi& epi, hipStream_t st) {
  if (tp < 32 || (tp & 31) || (n_in & 15) || (n_out & 31)) return TRJ_ERR_BAD_SHAPE;
  GemmPlan g = plan_gemm(tp, n_in, n_out, split_k);
  if (tp % (32 * g.mt) != 0) return TRJ_ERR_BAD_SHAPE;
#define TRJ_P(M)                                                                             \
  do {                                                                                       \
    if (g.rt == 1) launch_p<M, 1, 8, Epi>(xp, w, tp, n_in, n_out, g.split_k, epi, st);           \
    else if (g.rt == 3) launch_p<M, 3, 2, Epi>(xp, w, tp, n_in, n_out, g.split_k, epi, st);      \
    else if (g.rt == 4 && g.kw == 2) launch_p<M, 4, 2, Epi>(xp, w, tp, n_in, n_out, g.split_k, epi, st); \
    else if (g.rt == 4) launch_p<M, 4, 1, Epi>(xp, w, tp, n_in, n_out, g.split_k, epi, st);       \
    else if (g.kw == 4) launch_p<M, 2, 4, Epi>(xp, w, tp, n_in, n_out, g.split_k, epi, st);  \
    else launch_p<M, 2, 2, Epi>(xp, w, tp, n_in, n_out, g.split_k, epi, st);                 \
  } while (0)
  if (g.big && g.wt == 4) launch_t<4, 4, 4, Epi>(xp, w, tp, n_in, n_out, g.split_k, epi, st);
  else if (g.big) launch_t<4, 4, 2, Epi>(xp, w, tp, n_in, n_out, g.split_k, epi, st);
  else if (g.mt == 1) TRJ_P(1); else if (g.mt == 2) TRJ_P(2); else if (g.mt == 3) TRJ_P(3); else TRJ_P(4);
#undef TRJ_P
  return check_launch();
}

// the launch plan of a projection as six numbers (for tests and experiments): row-tile
// columns per pass, row tiles and k-parts per workgroup, row tiles per wavefront, grid
// k-splits, 1 if the many-rows kernel runs
void gemm_bf16_describe_plan(int tp, int n_in, int n_out, int split_k, int32_t out[6]) {
  GemmPlan g = plan_gemm(tp, n_in, n_out, split_k);
  out[0] = g.mt; out[1] = g.rt; out[2] = g.kw; out[3] = g.big ? g.wt : 1; out[4] = g.split_k;
  out[5] = g.big ? 1 : 0;
}

// number of grid splits a request for split_k really gets
int gemm_bf16_clamp_split(int n_out, int tp, int n_in, int split_k) {
  return plan_gemm(tp, n_in, n_out, split_k).split_k;
}

int gemm_bf16_split_k(int n_out, int tp, int n_in) {
  // projections whose epilogue is a plain partial-sum store are split along k until the
  // launch has about one workgroup (of 2 row tiles) per compute unit
  int mt = tp <= 96 ? tp / 32 : 4;
  int groups = ((n_out / 32 + 1) / 2) * (tp / (32 * mt));
  if (mt == 4 && tune().gemm_big_t > 0 && tp >= tune().gemm_big_t)
    groups = ((n_out / 32 + 7) / 8) * (tp / 128);  // 8 row tiles per workgroup there
  // up to 64 token rows twice as many splits pay: the launch then takes the (4 row tiles,
  // 1 k-part) shape, whose workgroups re-read half as much of the activations (down
  // 21.8 -> 20.2 us, output projection 10.8 -> 10.3 us, the sum over 8 partials instead of
  // 4 costs 0.3 us; step -1.3 % at 1..64 rows, +1 % at 96, +4 % at 128 rows)
  const int target = tp <= 64 ? 2 * tune().gemm_target_wgs : tune().gemm_target_wgs;
  int sk = (target + groups - 1) / groups;
  if (sk > tune().max_split_k) sk = tune().max_split_k;
  return gemm_bf16_clamp_split(n_out, tp, n_in, sk);
}

int launch_gemm_store_f32(const uint16_t* xp, const uint16_t* w, int T, int tp, int n_in,
                          int n_out, int split_k, const RowScale& rs, float* y, hipStream_t st) {
  if (rs.ssq) {
    EpiStoreF32T<true> e{rs, y, n_out, T, (size_t)T * n_out};
    return launch_gemm(xp, w, tp, n_in, n_out, split_k, e, st);
  }
  EpiStoreF32T<false> e{rs, y, n_out, T, (size_t)T * n_out};
  return launch_gemm(xp, w, tp, n_in, n_out, split_k, e, st);
}

// LM head with the argmax taken in the epilogue: argmax_out[t] = lowest index of the row
// maximum of x W^T; cand: T * n_out / 32 candidates of scratch
__global__ __launch_bounds__(256) void argmax_cand_kernel(const ArgmaxCand* __restrict__ cand,
                                                          int n_tiles, int32_t* __restrict__ out) {
  const ArgmaxCand* row = cand + (size_t)blockIdx.x * n_tiles;
  float bv = -INFINITY;
  int bi = INT32_MAX;
  for (int j = threadIdx.x; j < n_tiles; j += 256) {
    const ArgmaxCand c = row[j];
    if (c.v > bv || (c.v == bv && c.i < bi)) { bv = c.v; bi = c.i; }
  }
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(bv, o);
    const int oi = __shfl_xor(bi, o);
    if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
  }
  __shared__ float sv[4];
  __shared__ int si[4];
  if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w)
      if (sv[w] > bv || (sv[w] == bv && si[w] < bi)) { bv = sv[w]; bi = si[w]; }
    out[blockIdx.x] = bi == INT32_MAX ? 0 : bi;
  }
}
size_t gemm_lm_argmax_scratch_bytes(int T, int n_out) { return (size_t)T * (n_out / 32) * sizeof(ArgmaxCand); }
int launch_gemm_lm_argmax(const uint16_t* xp, const uint16_t* w, int T, int tp, int n_in, int n_out,
                          const RowScale& rs, void* cand, int32_t* argmax_out, hipStream_t st) {
  EpiArgmax e{rs, static_cast<ArgmaxCand*>(cand), T, n_out / 32};
  int rc = launch_gemm(xp, w, tp, n_in, n_out, 1, e, st);
  if (rc != TRJ_OK) return rc;
  argmax_cand_kernel<<<T, 256, 0, st>>>(static_cast<const ArgmaxCand*>(cand), n_out / 32, argmax_out);
  return check_launch();
}

int launch_gemm_gate_up(const uint16_t* xp, const uint16_t* w, int tp, int n_in, int d_ffn,
                        const RowScale& rs, uint16_t* act, hipStream_t st) {
  EpiGateUp e{rs, act, tp};
  return launch_gemm(xp, w, tp, n_in, 2 * d_ffn, 1, e, st);
}

int launch_gemm_qkv(const uint16_t* xp, const uint16_t* w, int T, int tp, int n_in, int n_heads,
                    int n_kv_heads, int dh, int s_pool, const RowScale& rs, const float2* cs,
                    const int32_t* cs_row, const int32_t* row_slot, uint16_t* q, uint16_t* k_layer,
                    uint16_t* v_layer, hipStream_t st) {
  EpiQKV e{rs, cs, cs_row, row_slot, q, k_layer, v_layer, T, n_heads, n_kv_heads, dh, s_pool};
  return launch_gemm(xp, w, tp, n_in, (n_heads + 2 * n_kv_heads) * dh, 1, e, st);
}

// ------------------------------------------------------------------ split-k sum + residual + norm input
// x[t] += sum_s partial[s][t] (fixed order: s = 0, 1, ...), and the next projection's input
// bf16(x * g) in the tiled activation layout, NOT yet divided by the row's norm: each
// workgroup owns one column part (about 1024 columns) of one token row and writes that part's sum of x^2 to
// ssq[part][t]; the consuming projection divides (RowScale).  Rows t >= T of the padded tile
// are written as zeros.  Without partials the row comes from the embedding table instead
// (x[t] = E[tok[t]], ids outside [0, vocab) clamped).
constexpr int RN_MAX_THREADS = 256, RN_SB = 8;
// column parts of a row: about 1024 columns each, at most RS_MAX_PARTS
int reduce_norm_parts(int d) {
  int p = (d + 1023) / 1024;
  return p > RS_MAX_PARTS ? RS_MAX_PARTS : p;
}
// threads per workgroup (8 columns each): the part's share of the row, in whole wavefronts
static int reduce_norm_threads(int d) {
  const int ngran = d >> 3, parts = reduce_norm_parts(d);
  return ((ngran + parts - 1) / parts + WAVE - 1) / WAVE * WAVE;
}

// a, b += partial sums of splits 0 .. n_split-1 in that order, SB loads in flight at a time
// (indices past the last split are clamped for the load and left out of the sum)
template <int SB>
__device__ __forceinline__ void add_splits(const float* __restrict__ pr, int n_split,
                                           size_t split_stride, f32x4& a, f32x4& b) {
  for (int s0 = 0; s0 < n_split; s0 += SB) {
    f32x4 pa[SB], pb[SB];
#pragma unroll
    for (int j = 0; j < SB; ++j) {
      const float* q = pr + min(s0 + j, n_split - 1) * split_stride;
      pa[j] = *reinterpret_cast<const f32x4*>(q);
      pb[j] = *reinterpret_cast<const f32x4*>(q + 4);
    }
#pragma unroll
    for (int j = 0; j < SB; ++j) {
      if (s0 + j < n_split) {
        a += pa[j];
        b += pb[j];
      }
    }
  }
}

__global__ __launch_bounds__(RN_MAX_THREADS) void reduce_norm_kernel(
    const float* __restrict__ partial, int n_split, size_t split_stride, float* __restrict__ x,
    const uint16_t* __restrict__ embed, const int32_t* __restrict__ tok, int vocab,
    const float* __restrict__ g, int T, int d, int tp, uint16_t* __restrict__ hp,
    float* __restrict__ ssq) {
  const int t = blockIdx.x, part = blockIdx.y, tid = threadIdx.x;
  const int ngran = d >> 3;
  const int gi_raw = part * blockDim.x + tid;
  const bool live = gi_raw < ngran;
  const int gi = min(gi_raw, ngran - 1);
  if (t >= T) {
    const u32x4 z = {0, 0, 0, 0};
    if (live) *reinterpret_cast<u32x4*>(hp + a_off(t, gi * 8, tp)) = z;
    if (tid == 0) ssq[(size_t)part * tp + t] = 0.f;
    return;
  }
  // every load of the thread is issued before the first one is used
  float* xr = x + (size_t)t * d + gi * 8;
  f32x4 a, b;
  const f32x4 g0 = *reinterpret_cast<const f32x4*>(g + gi * 8);
  const f32x4 g1 = *reinterpret_cast<const f32x4*>(g + gi * 8 + 4);
  if (embed) {  // uniform over the launch
    int id = tok[t];
    id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
    const u32x4 v = *reinterpret_cast<const u32x4*>(embed + (size_t)id * d + gi * 8);
    a = f32x4{__builtin_bit_cast(float, v[0] << 16), __builtin_bit_cast(float, v[0] & 0xffff0000u),
              __builtin_bit_cast(float, v[1] << 16), __builtin_bit_cast(float, v[1] & 0xffff0000u)};
    b = f32x4{__builtin_bit_cast(float, v[2] << 16), __builtin_bit_cast(float, v[2] & 0xffff0000u),
              __builtin_bit_cast(float, v[3] << 16), __builtin_bit_cast(float, v[3] & 0xffff0000u)};
  } else {
    a = *reinterpret_cast<f32x4*>(xr);
    b = *reinterpret_cast<f32x4*>(xr + 4);
    // as many loads in flight as there are splits, up to RN_SB (n_split is uniform over
    // the launch); the sum runs in the same order s = 0, 1, ... whichever batch is taken
    const float* pr = partial + (size_t)t * d + gi * 8;
    if (n_split <= 2) add_splits<2>(pr, n_split, split_stride, a, b);
    else if (n_split <= 4) add_splits<4>(pr, n_split, split_stride, a, b);
    else add_splits<RN_SB>(pr, n_split, split_stride, a, b);
  }
  float ss = 0.f;
  if (live) {
    if (embed || n_split > 0) {
      *reinterpret_cast<f32x4*>(xr) = a;
      *reinterpret_cast<f32x4*>(xr + 4) = b;
    }
    u32x4 pk = {pack2bf(a[0] * g0[0], a[1] * g0[1]), pack2bf(a[2] * g0[2], a[3] * g0[3]),
                pack2bf(b[0] * g1[0], b[1] * g1[1]), pack2bf(b[2] * g1[2], b[3] * g1[3])};
    *reinterpret_cast<u32x4*>(hp + a_off(t, gi * 8, tp)) = pk;
#pragma unroll
    for (int e = 0; e < 4; ++e) ss += a[e] * a[e] + b[e] * b[e];
  }
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
  __shared__ float wsum[RN_MAX_THREADS / WAVE];
  if ((tid & 63) == 0) wsum[tid >> 6] = ss;
  __syncthreads();
  if (tid == 0) {
    float tot = 0.f;
    for (int w = 0; w < (int)blockDim.x / WAVE; ++w) tot += wsum[w];
    ssq[(size_t)part * tp + t] = tot;
  }
}

int launch_reduce_norm(const float* partial, int n_split, float* x, const float* g, int T, int d,
                       int tp, uint16_t* hp, float* ssq, hipStream_t st) {
  if ((d & 7) || reduce_norm_threads(d) > RN_MAX_THREADS) return TRJ_ERR_BAD_SHAPE;
  reduce_norm_kernel<<<dim3(tp, reduce_norm_parts(d)), reduce_norm_threads(d), 0, st>>>(
      partial, n_split, (size_t)T * d, x, nullptr, nullptr, 0, g, T, d, tp, hp, ssq);
  return check_launch();
}

int launch_embed_norm(const uint16_t* embed, const int32_t* tok, int T, int d, int vocab, float* x,
                      const float* g, int tp, uint16_t* hp, float* ssq, hipStream_t st) {
  if ((d & 7) || reduce_norm_threads(d) > RN_MAX_THREADS) return TRJ_ERR_BAD_SHAPE;
  reduce_norm_kernel<<<dim3(tp, reduce_norm_parts(d)), reduce_norm_threads(d), 0, st>>>(
      nullptr, 0, 0, x, embed, tok, vocab, g, T, d, tp, hp, ssq);
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
