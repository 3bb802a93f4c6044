// Backward of the fused two-layer ReLU MLPs of the encoder (Section 3.3.4: one back-propagation
// through the GNN of Section 3.4), per tile of 32 rows per wave, all contractions on the matrix
// cores. For y = relu(relu(x W1 + b1) W2 + b2) and upstream dy:
//     dz2 = dy * [y > 0],  dz1 = (dz2 W2^T) * [z1 > 0],  dx = dz1 W1^T.
// Everything is kept transposed (features x rows: lane = row, registers = features), so each
// result is already laid out as the next contraction's B operand:
//     z1^T  = W1^T x^T            (as in the forward kernel)
//     y^T   = W2^T z1^T           (EDGE only: its per-edge output is not stored by the forward)
//     dz1^T = W2 dz2^T            (W2 pre-arranged with the contraction over its columns)
//     dx^T  = W1 dz1^T            (W1 pre-arranged with the contraction over its columns)
// Weights: a block of 4 waves (128 rows) walks through the four weight matrices in units of
// H / 16 fragments (1 KB each; the fragments one 32-feature output block needs), four units to a
// group; in the bf16 instantiations a group is fetched from L2 once per block -- each wave a
// quarter of it, requested a whole group (about 2000 MFMA cycles at H = 256) before it is needed
// -- into a double-buffered LDS area and read from there by all four waves, one block barrier per
// group (fetching every fragment per wave made the kernel L2-bound: 780 KB of weights per 32
// rows at H = 256; groups of one unit left the fetch latency exposed). The fp32 instantiations
// read their fragments straight from L2.
// The kernel writes z1, dz1, dz2 as [rows, H] for the weight-gradient kernel, and dx:
//   EDGE: per-edge gradients w.r.t. h_sender and h_receiver ([E, H] each; summed per node later),
//   NODE: d/dh and d/dagg [N, H],   EMBED: nothing (its inputs are data).
// Gradients w.r.t. node states travel between kernels in the operand type: their only readers
// are this kernel's instantiations, which turn them into operands of that type anyway, and the
// per-node gather, which sums in fp32.
#pragma once
#include <type_traits>
#include "mlp2.hip.h"

struct Mlp2BwdArgs {
  int64_t n_rows, n_blocks;
  const void *W1s, *W2s;     // forward fragment order
  const void *W2bt, *W1bt;   // contraction over the weight's columns (see swizzle_chain)
  const float *b1, *b2;
  int nslab1;
  const void *h, *agg;       // forward inputs, operand type
  const int32_t *agg_src;    // NODE: [N] row of agg per node, -1 = none (zeros are read); or nullptr
  const void *zero_row;      // 1 KB of zeros
  const void *y;             // saved forward output [N, H] operand type      (NODE, EMBED)
  const void *dy;            // upstream gradient [N, H], operand type (EDGE: indexed by receiver)
  const int32_t *in_ptr, *in_src, *in_dst;
  const float *edge_feat;
  const int32_t *node_op;
  const float *node_dense;
  int De, Tn, Dd;
  void *z1, *dz1, *dz2;      // [rows, H] operand type
  void *dx_a, *dx_b;         // EDGE: d h_sender, d h_receiver [E, H] operand type;
                             // NODE: d h, d agg [N, H] operand type
};

// Accumulator tile (features x rows) -> the 32 / (2V) operand slabs of its 32 features.
template <typename T>
__device__ __forceinline__ typename Operand<T>::vec acc_slab(const f32x16 &acc, int q);
template <>
__device__ __forceinline__ f32x4 acc_slab<float>(const f32x16 &acc, int q) {
  return f32x4{acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
}
template <>
__device__ __forceinline__ bf16x8 acc_slab<bf16_t>(const f32x16 &acc, int q) {
  return pack_bf16x8(acc[8 * q], acc[8 * q + 1], acc[8 * q + 2], acc[8 * q + 3], acc[8 * q + 4],
                     acc[8 * q + 5], acc[8 * q + 6], acc[8 * q + 7]);
}

// Weight fragments for all four waves, UG units of UF fragments per group. SHARED: through LDS
// (see the file header); otherwise each wave reads its own from global memory. `idx(u, j)` is
// the index inside W (already offset by the lane) of fragment j of the group's u-th unit, or
// negative if there is no such fragment.
template <typename vecT, int UF, int UG, bool SHARED>
struct WeightGroups {
  static constexpr int GF = UF * UG, PW = GF / 4;         // fragments per group / fetched per wave
  static_assert(GF % 4 == 0, "a group is fetched by four waves");
  f32x4 (*buf)[GF][64];                                   // [2][GF][64] in LDS (SHARED)
  int p = 0, wave, lane;
  f32x4 r[PW];
  template <typename Idx>
  __device__ __forceinline__ void fetch(const vecT *W, Idx idx) {
    if constexpr (SHARED) {
#pragma unroll
      for (int i = 0; i < PW; ++i) {
        const int jg = wave * PW + i;
        const int fi = idx(jg / UF, jg % UF);
        if (fi >= 0) r[i] = __builtin_bit_cast(f32x4, W[(size_t)fi * 64]);
      }
    }
  }
  __device__ __forceinline__ void commit(int q) {
    if constexpr (SHARED) {
#pragma unroll
      for (int i = 0; i < PW; ++i) buf[q][wave * PW + i][lane] = r[i];
    }
  }
  // first group of a phase: fetch, store, barrier
  template <typename Idx>
  __device__ __forceinline__ void begin(const vecT *W, Idx idx) {
    if constexpr (SHARED) {
      fetch(W, idx);
      commit(p);
      __syncthreads();
    }
  }
  // after the MFMAs of the current group: publish the next one (already fetched), swap
  __device__ __forceinline__ void next(bool have_next) {
    if constexpr (SHARED) {
      if (have_next) commit(p ^ 1);
      __syncthreads();
      p ^= 1;
    }
  }
  // fragment j of unit u of the current group
  template <typename Idx>
  __device__ __forceinline__ vecT get(const vecT *W, Idx idx, int u, int j) const {
    if constexpr (SHARED) return __builtin_bit_cast(vecT, buf[p][u * UF + j][lane]);
    else return W[(size_t)idx(u, j) * 64];
  }
};

// One unit's fragments as registers (SHARED: all LDS reads in flight together, the MFMAs behind
// them wait for one fragment each) or, for the direct path, read where they are used.
template <typename vecT, int UF, int UG, bool SHARED>
struct UnitFrags {
  vecT w[SHARED ? UF : 1];
  template <typename Idx>
  __device__ __forceinline__ void load(const WeightGroups<vecT, UF, UG, SHARED> &wg, const vecT *W, Idx idx, int u) {
    if constexpr (SHARED) {
#pragma unroll
      for (int j = 0; j < UF; ++j) w[j] = wg.get(W, idx, u, j);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  template <typename Idx>
  __device__ __forceinline__ vecT operator()(const WeightGroups<vecT, UF, UG, SHARED> &wg, const vecT *W, Idx idx,
                                             int u, int j) const {
    if constexpr (SHARED) return w[j];
    else return wg.get(W, idx, u, j);
  }
};

template <typename T1, typename T, int H, int KIND>
__global__ __launch_bounds__(256) void mlp2_bwd_kernel(const Mlp2BwdArgs a) {
  using Opd = Operand<T>;
  using vec = typename Opd::vec;
  constexpr int V = Opd::V, SL = 2 * V, MB = H / 32, HS = H / SL, QB = 32 / SL;
  using Opd1 = Operand<T1>;
  using vec1 = typename Opd1::vec;
  constexpr int V1 = Opd1::V, SL1 = 2 * V1;
  constexpr bool SHARED = sizeof(T) == 2;
  constexpr int UF = MB * QB;                               // fragments per unit (H / 16 in bf16)
  constexpr int SPU = UF / MB;                              // layer-1 slabs per unit
  constexpr int UG = H >= 256 ? 4 : 2;                      // units per group (H <= 128: two blocks share a CU's LDS)
  using WG = WeightGroups<vec, UF, UG, SHARED>;
  using UFr = UnitFrags<vec, UF, UG, SHARED>;

  const int64_t per_xcd = (a.n_blocks + 7) / 8;
  const int64_t tile = (int64_t)(blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (tile >= a.n_blocks) return;                           // (the whole block)
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, g = lane >> 5;
  const int64_t row0 = (tile * 4 + wave) * 32;
  int64_t row = row0 + l32;
  const bool valid = row < a.n_rows;
  if (!valid) row = a.n_rows - 1;
  // every [rows, H] result leaves through a per-wave staging buffer, one 32-feature block at a time
  extern __shared__ __align__(16) char smem[];
  char *stage = smem + wave * BlockStage<float>::BYTES;
  const int64_t left = a.n_rows - row0;
  const int n_valid = left < 32 ? (left > 0 ? (int)left : 0) : 32;
  WG wg;
  wg.buf = reinterpret_cast<f32x4 (*)[WG::GF][64]>(smem + 4 * BlockStage<float>::BYTES);
  wg.wave = wave; wg.lane = lane;

  // ---------------- z1^T = relu(W1^T x^T + b1), exactly as in the forward kernel
  f32x16 acc1[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc1[mb][r] = a.b1[32 * mb + acc_row(r, g)];
  int64_t src = 0, dst = 0;
  {
    // layer 1's fragments are contiguous: unit u = fragments [u * UF, u * UF + UF) = SPU slabs
    const vec *W1 = (const vec *)a.W1s + lane;              // (vec and vec1 are both 16 bytes)
    const int n_frag = a.nslab1 * MB, n_units = (a.nslab1 + SPU - 1) / SPU;
    [[maybe_unused]] const T *pa = nullptr, *pb = nullptr;
    [[maybe_unused]] EmbedRow er;
    if constexpr (KIND == KIND_EDGE) {
      src = a.in_src[row];
      dst = a.in_dst[row];
      pa = (const T *)a.h + (size_t)src * H + g * V;
      pb = (const T *)a.h + (size_t)dst * H + g * V;
    } else if constexpr (KIND == KIND_NODE) {
      pa = (const T *)a.h + (size_t)row * H + g * V;
      const int64_t ar = a.agg_src ? (int64_t)a.agg_src[row] : row;
      pb = ar < 0 ? (const T *)a.zero_row + g * V : (const T *)a.agg + (size_t)ar * H + g * V;
    } else {
      er = load_embed_row(a.node_op, a.in_ptr, a.node_dense, a.Dd, row);
    }
    // fragment j of unit u of the group that starts at unit u0
    auto idx_from = [&](int u0) {
      return [=](int u, int j) { const int f = (u0 + u) * UF + j; return f < n_frag ? f : -1; };
    };
    wg.begin(W1, idx_from(0));
    int u0 = 0;
    if constexpr (KIND != KIND_EMBED) {
      // the 2 HS slabs of the two H-wide input parts: gathered rows, requested XQ slabs ahead
      constexpr int NSH = 2 * HS, XQ = 8 < NSH ? 8 : NSH, NSU = NSH / SPU;
      static_assert(NSU % UG == 0, "the H-wide parts fill whole groups");
      auto load_slab = [&](int s) -> vec {
        if (s < HS) return *(const vec *)(pa + s * SL);
        return *(const vec *)(pb + (s - HS) * SL);   // (the forward zeroed the received sums of nodes without in-edges)
      };
      vec xq[XQ];
#pragma unroll
      for (int s = 0; s < XQ; ++s) xq[s] = load_slab(s);
#pragma unroll
      for (int g0 = 0; g0 < NSU; g0 += UG) {
        const auto idx = idx_from(g0);
        if (g0 + UG < n_units) wg.fetch(W1, idx_from(g0 + UG));
#pragma unroll
        for (int u = 0; u < UG; ++u) {
          UFr w;
          w.load(wg, W1, idx, u);
#pragma unroll
          for (int j2 = 0; j2 < SPU; ++j2) {
            const int sl = (g0 + u) * SPU + j2;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) Opd::mma(w(wg, W1, idx, u, j2 * MB + mb), xq[sl % XQ], acc1[mb]);
            if (sl + XQ < NSH) xq[sl % XQ] = load_slab(sl + XQ);
          }
        }
        wg.next(g0 + UG < n_units);
      }
      u0 = NSU;
    }
    // the remaining slabs (EDGE: edge attributes; EMBED: all of them)
    for (; u0 < n_units; u0 += UG) {
      const auto idx = idx_from(u0);
      if (u0 + UG < n_units) wg.fetch(W1, idx_from(u0 + UG));
#pragma unroll
      for (int u = 0; u < UG; ++u)
#pragma unroll
        for (int j2 = 0; j2 < SPU; ++j2) {
          const int sl = (u0 + u) * SPU + j2;
          if (sl < a.nslab1) {
            if constexpr (KIND == KIND_EMBED) {
              vec1 x;
#pragma unroll
              for (int j = 0; j < V1; ++j) {
                const int k = sl * SL1 + g * V1 + j;        // column of [edge-attr sum | one-hot | dense]
                float v = 0.f;
                if (k >= a.De && k < a.De + a.Tn) v = (k - a.De == er.op) ? 1.f : 0.f;
                else if (k >= a.De + a.Tn && k < a.De + a.Tn + a.Dd) v = er.dense[k - a.De - a.Tn];
                x[j] = Opd1::from_float(v);
              }
              if (sl * SL1 + g * V1 < a.De) {               // (De and V1 are multiples of 4)
                const f32x4 e4 = embed_columns(er, a.edge_feat, a.De, 0, sl * SL1 + g * V1);
#pragma unroll
                for (int j = 0; j < 4; ++j) x[j] = Opd1::from_float(e4[j]);
              }
#pragma unroll
              for (int mb = 0; mb < MB; ++mb)
                Opd1::mma(__builtin_bit_cast(vec1, wg.get(W1, idx, u, j2 * MB + mb)), x, acc1[mb]);
            } else {
              const vec x = tail_to_operand<T>(load_tail<V>(a.edge_feat + (size_t)row * a.De, a.De, sl - 2 * HS, g));
#pragma unroll
              for (int mb = 0; mb < MB; ++mb) Opd::mma(wg.get(W1, idx, u, j2 * MB + mb), x, acc1[mb]);
            }
          }
        }
      wg.next(u0 + UG < n_units);
    }
  }
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
    for (int r = 0; r < 16; ++r) acc1[mb][r] = relu_f32(acc1[mb][r]);
    store_block_via_lds<T, H>((T *)a.z1, row0, n_valid, mb, lane, acc1[mb], stage);
  }

  // ---------------- dz2^T = dy^T * [y^T > 0], stored and kept as operand slabs
  vec dz2s[MB][QB];
  {
    using DY = T;
    const DY *dyrow = (const DY *)a.dy + (size_t)(KIND == KIND_EDGE ? dst : row) * H;
    [[maybe_unused]] const vec *W2 = (const vec *)a.W2s + lane;
    [[maybe_unused]] const T *yrow = KIND == KIND_EDGE ? nullptr : (const T *)a.y + (size_t)row * H + 4 * g;
    // dy (and, where the forward stored it, y) of block nb + 1 is requested while block nb is
    // worked on: the fences of the staged stores keep the compiler from doing that itself
    auto load_dy = [&](int nb, f32x16 &d, f32x16 &yv) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float v[4];
        load4<DY>(dyrow + 32 * nb + 8 * q + 4 * g, v);
        d[4 * q] = v[0]; d[4 * q + 1] = v[1]; d[4 * q + 2] = v[2]; d[4 * q + 3] = v[3];
        if constexpr (KIND != KIND_EDGE) {
          load4<T>(yrow + 32 * nb + 8 * q, v);
          yv[4 * q] = v[0]; yv[4 * q + 1] = v[1]; yv[4 * q + 2] = v[2]; yv[4 * q + 3] = v[3];
        }
      }
    };
    f32x16 dyc, yc, dyn, yn;
    load_dy(0, dyc, yc);
    // EDGE: y^T block nb needs W2's fragments ((mb, q), nb) for all (mb, q): unit nb
    auto idx_from = [&](int u0) { return [=](int u, int j) { return j * MB + u0 + u; }; };
    if constexpr (KIND == KIND_EDGE) wg.begin(W2, idx_from(0));
#pragma unroll
    for (int nb = 0; nb < MB; ++nb) {
      if (nb + 1 < MB) load_dy(nb + 1, dyn, yn);
      if constexpr (KIND == KIND_EDGE) {
        const int g0 = nb / UG * UG, u = nb % UG;
        const auto idx = idx_from(g0);
        if (u == 0 && g0 + UG < MB) wg.fetch(W2, idx_from(g0 + UG));
        UFr w;
        w.load(wg, W2, idx, u);
#pragma unroll
        for (int r = 0; r < 16; ++r) yc[r] = a.b2[32 * nb + acc_row(r, g)];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
          for (int q = 0; q < QB; ++q) Opd::mma(w(wg, W2, idx, u, mb * QB + q), acc_slab<T>(acc1[mb], q), yc);
        if (u == UG - 1) wg.next(g0 + UG < MB);
      }
      f32x16 d;
#pragma unroll
      for (int r = 0; r < 16; ++r) d[r] = yc[r] > 0.f ? dyc[r] : 0.f;
      store_block_via_lds<T, H>((T *)a.dz2, row0, n_valid, nb, lane, d, stage);
#pragma unroll
      for (int q = 0; q < QB; ++q) dz2s[nb][q] = acc_slab<T>(d, q);
      if (nb + 1 < MB) { dyc = dyn; yc = yn; }
    }
  }

  // ---------------- dz1^T = (W2 dz2^T) * [z1^T > 0]: unit mb = the W2^T fragments of block mb
  vec dz1s[MB][QB];
  {
    const vec *W2b = (const vec *)a.W2bt + lane;
    auto idx_from = [&](int u0) { return [=](int u, int j) { return j * MB + u0 + u; }; };
    wg.begin(W2b, idx_from(0));
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int g0 = mb / UG * UG, u = mb % UG;
      const auto idx = idx_from(g0);
      if (u == 0 && g0 + UG < MB) wg.fetch(W2b, idx_from(g0 + UG));
      UFr w;
      w.load(wg, W2b, idx, u);
      f32x16 d;
#pragma unroll
      for (int r = 0; r < 16; ++r) d[r] = 0.f;
#pragma unroll
      for (int nb = 0; nb < MB; ++nb)
#pragma unroll
        for (int q = 0; q < QB; ++q) Opd::mma(w(wg, W2b, idx, u, nb * QB + q), dz2s[nb][q], d);
      if (u == UG - 1) wg.next(g0 + UG < MB);
#pragma unroll
      for (int r = 0; r < 16; ++r) d[r] = acc1[mb][r] > 0.f ? d[r] : 0.f;
      store_block_via_lds<T, H>((T *)a.dz1, row0, n_valid, mb, lane, d, stage);
#pragma unroll
      for (int q = 0; q < QB; ++q) dz1s[mb][q] = acc_slab<T>(d, q);
    }
  }

  // ---------------- dx^T = W1 dz1^T over the first 2H input columns (h parts only): unit kb =
  // the W1^T fragments of the 32-column block kb of [part a | part b]
  if constexpr (KIND != KIND_EMBED) {
    const vec *W1b = (const vec *)a.W1bt + lane;
    constexpr int KB = 2 * MB;
    auto idx_from = [&](int u0) { return [=](int u, int j) { return j * KB + u0 + u; }; };
    wg.begin(W1b, idx_from(0));
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
      const int g0 = kb / UG * UG, u = kb % UG;
      const auto idx = idx_from(g0);
      if (u == 0 && g0 + UG < KB) wg.fetch(W1b, idx_from(g0 + UG));
      UFr w;
      w.load(wg, W1b, idx, u);
      f32x16 d;
#pragma unroll
      for (int r = 0; r < 16; ++r) d[r] = 0.f;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int q = 0; q < QB; ++q) Opd::mma(w(wg, W1b, idx, u, mb * QB + q), dz1s[mb][q], d);
      if (u == UG - 1) wg.next(g0 + UG < KB);
      if constexpr (KIND == KIND_EDGE) {
        T *o = (T *)(kb < MB ? a.dx_a : a.dx_b);
        store_block_via_lds<T, H>(o, row0, n_valid, kb % MB, lane, d, stage);
      } else {
        store_block_via_lds<T, H>((T *)(kb < MB ? a.dx_a : a.dx_b), row0, n_valid, kb % MB, lane, d, stage);
      }
    }
  }
}

// dynamic LDS of mlp2_bwd_kernel: four staging buffers, then (bf16) two groups of fragments
template <typename T, int H>
constexpr size_t mlp2_bwd_lds_bytes() {
  constexpr int MB = H / 32, QB = 32 / (2 * Operand<T>::V), UG = H >= 256 ? 4 : 2;
  return 4 * (size_t)BlockStage<float>::BYTES + (sizeof(T) == 2 ? 2 * (size_t)(MB * QB * UG) * 1024 : 0);
}
