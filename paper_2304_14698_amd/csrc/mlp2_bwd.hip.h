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
// Weights: a block of 4 waves (128 rows) walks through the four weight matrices in groups of
// H / 16 fragments (1 KB each); in the bf16 instantiations a group is fetched from L2 once per
// block -- each wave a quarter of it -- into a double-buffered LDS area and read from there by
// all four waves, one block barrier per group (fetching every fragment per wave made the kernel
// L2-bound: 780 KB of weights per 32 rows at H = 256). The fp32 instantiations read their
// fragments straight from L2.
// The kernel writes z1, dz1, dz2 as [rows, H] for the weight-gradient kernel, and dx:
//   EDGE: per-edge gradients w.r.t. h_sender and h_receiver ([E, H] each; summed per node later),
//   NODE: d/dh [N, H] and d/dagg [N, H] (fp32),   EMBED: nothing (its inputs are data).
#pragma once
#include "mlp2.hip.h"

struct Mlp2BwdArgs {
  int64_t n_rows, n_blocks;
  const void *W1s, *W2s;     // forward fragment order
  const void *W2bt, *W1bt;   // contraction over the weight's columns (see swizzle_chain)
  const float *b1, *b2;
  int nslab1;
  const void *h, *agg;       // forward inputs, operand type
  const void *y;             // saved forward output [N, H] operand type      (NODE, EMBED)
  const float *dy;           // upstream gradient: [N, H] fp32 (EDGE: indexed by receiver)
  const int32_t *in_ptr, *in_src, *in_dst;
  const float *edge_feat;
  const int32_t *node_op;
  const float *node_dense;
  int De, Tn, Dd;
  void *z1, *dz1, *dz2;      // [rows, H] operand type
  void *dx_a, *dx_b;         // EDGE: d h_sender, d h_receiver [E, H] operand type;
                             // NODE: d h, d agg [N, H] fp32
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

// Weight fragments of one group for all four waves. SHARED: through LDS (see the file header);
// otherwise each wave reads its own from global memory. `idx(j)` is the fragment index of the
// group's j-th fragment inside W (already offset by the lane), `n_valid` how many exist.
template <typename vecT, int GF, bool SHARED>
struct WeightGroups {
  static constexpr int PW = GF / 4 > 0 ? GF / 4 : 1;      // fragments a wave fetches per group
  f32x4 (*buf)[GF][64];                                   // [2][GF][64] in LDS (SHARED)
  int p = 0, wave, lane;
  f32x4 r[PW];
  template <typename Idx>
  __device__ __forceinline__ void fetch(const vecT *W, Idx idx, int n_valid) {
    if constexpr (SHARED) {
#pragma unroll
      for (int i = 0; i < PW; ++i) {
        const int j = wave * PW + i;
        if (j < GF && j < n_valid) r[i] = __builtin_bit_cast(f32x4, W[(size_t)idx(j) * 64]);
      }
    }
  }
  __device__ __forceinline__ void commit(int q) {
    if constexpr (SHARED) {
#pragma unroll
      for (int i = 0; i < PW; ++i) {
        const int j = wave * PW + i;
        if (j < GF) buf[q][j][lane] = r[i];
      }
    }
  }
  // first group of a phase: fetch, store, barrier
  template <typename Idx>
  __device__ __forceinline__ void begin(const vecT *W, Idx idx, int n_valid) {
    if constexpr (SHARED) {
      fetch(W, idx, n_valid);
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
  template <typename Idx>
  __device__ __forceinline__ vecT get(const vecT *W, Idx idx, int j) const {
    if constexpr (SHARED) return __builtin_bit_cast(vecT, buf[p][j][lane]);
    else return W[(size_t)idx(j) * 64];
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
  constexpr int GF = MB * QB;                               // fragments per group (H / 16 in bf16)
  constexpr int SPG = GF / MB;                              // layer-1 slabs per group

  const int64_t per_xcd = (a.n_blocks + 7) / 8;
  const int64_t tile = (int64_t)(blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (tile >= a.n_blocks) return;                           // (the whole block)
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, g = lane >> 5;
  const int64_t row0 = (tile * 4 + wave) * 32;
  int64_t row = row0 + l32;
  const bool valid = row < a.n_rows;
  if (!valid) row = a.n_rows - 1;
  // every [rows, H] result leaves through a per-wave staging buffer, one 32-feature block at a time
  __shared__ __align__(16) char stage_all[4][BlockStage<float>::BYTES];
  __shared__ __align__(16) f32x4 wshared[SHARED ? 2 : 1][SHARED ? GF : 1][64];
  char *stage = stage_all[wave];
  const int64_t left = a.n_rows - row0;
  const int n_valid = left < 32 ? (left > 0 ? (int)left : 0) : 32;
  WeightGroups<vec, GF, SHARED> wg;
  wg.buf = reinterpret_cast<f32x4 (*)[GF][64]>(&wshared[0][0][0]); wg.wave = wave; wg.lane = lane;

  // ---------------- z1^T = relu(W1^T x^T + b1), exactly as in the forward kernel
  f32x16 acc1[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc1[mb][r] = a.b1[32 * mb + acc_row(r, g)];
  int64_t src = 0, dst = 0;
  {
    // layer 1's fragments are contiguous: group gi = fragments [gi * GF, gi * GF + GF) = SPG slabs
    const vec *W1 = (const vec *)a.W1s + lane;              // (vec and vec1 are both 16 bytes)
    const int n_frag = a.nslab1 * MB, n_groups = (a.nslab1 + SPG - 1) / SPG;
    [[maybe_unused]] const T *pa = nullptr, *pb = nullptr;
    [[maybe_unused]] bool has_in = true;
    [[maybe_unused]] EmbedRow er;
    if constexpr (KIND == KIND_EDGE) {
      src = a.in_src[row];
      dst = a.in_dst[row];
      pa = (const T *)a.h + (size_t)src * H + g * V;
      pb = (const T *)a.h + (size_t)dst * H + g * V;
    } else if constexpr (KIND == KIND_NODE) {
      pa = (const T *)a.h + (size_t)row * H + g * V;
      pb = (const T *)a.agg + (size_t)row * H + g * V;
      has_in = a.in_ptr[row + 1] > a.in_ptr[row];
    } else {
      er = load_embed_row(a.node_op, a.in_ptr, a.node_dense, a.Dd, row);
    }
    wg.begin(W1, [&](int j) { return j; }, n_frag);
    for (int gi = 0; gi < n_groups; ++gi) {
      const int f0 = gi * GF;
      if (gi + 1 < n_groups) wg.fetch(W1, [&](int j) { return f0 + GF + j; }, n_frag - f0 - GF);
#pragma unroll
      for (int j2 = 0; j2 < SPG; ++j2) {
        const int s = gi * SPG + j2;
        if (s < a.nslab1) {
          if constexpr (KIND == KIND_EMBED) {
            vec1 x;
#pragma unroll
            for (int j = 0; j < V1; ++j) {
              const int k = s * SL1 + g * V1 + j;           // column of [edge-attr sum | one-hot | dense]
              float v = 0.f;
              if (k >= a.De && k < a.De + a.Tn) v = (k - a.De == er.op) ? 1.f : 0.f;
              else if (k >= a.De + a.Tn && k < a.De + a.Tn + a.Dd) v = er.dense[k - a.De - a.Tn];
              x[j] = Opd1::from_float(v);
            }
            if (s * SL1 + g * V1 < a.De) {                  // (De and V1 are multiples of 4)
              const f32x4 e4 = embed_columns(er, a.edge_feat, a.De, 0, s * SL1 + g * V1);
#pragma unroll
              for (int j = 0; j < 4; ++j) x[j] = Opd1::from_float(e4[j]);
            }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
              Opd1::mma(__builtin_bit_cast(vec1, wg.get(W1, [&](int j) { return f0 + j; }, j2 * MB + mb)), x, acc1[mb]);
          } else {
            vec x;
            if (s < HS) x = *(const vec *)(pa + s * SL);
            else if (s < 2 * HS) x = has_in ? *(const vec *)(pb + (s - HS) * SL) : Opd::zero();
            else x = tail_to_operand<T>(load_tail<V>(a.edge_feat + (size_t)row * a.De, a.De, s - 2 * HS, g));
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
              Opd::mma(wg.get(W1, [&](int j) { return f0 + j; }, j2 * MB + mb), x, acc1[mb]);
          }
        }
      }
      wg.next(gi + 1 < n_groups);
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
    const float *dyrow = a.dy + (size_t)(KIND == KIND_EDGE ? dst : row) * H;
    [[maybe_unused]] const vec *W2 = (const vec *)a.W2s + lane;
    // EDGE: y^T block nb needs W2's fragments ((mb, q), nb) for all (mb, q): one group per nb
    if constexpr (KIND == KIND_EDGE) wg.begin(W2, [&](int j) { return j * MB; }, GF);
#pragma unroll
    for (int nb = 0; nb < MB; ++nb) {
      f32x16 yv;
      if constexpr (KIND == KIND_EDGE) {
        if (nb + 1 < MB) wg.fetch(W2, [&](int j) { return j * MB + nb + 1; }, GF);
#pragma unroll
        for (int r = 0; r < 16; ++r) yv[r] = a.b2[32 * nb + acc_row(r, g)];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
          for (int q = 0; q < QB; ++q)
            Opd::mma(wg.get(W2, [&](int j) { return j * MB + nb; }, mb * QB + q), acc_slab<T>(acc1[mb], q), yv);
        wg.next(nb + 1 < MB);
      } else {
        const T *yrow = (const T *)a.y + (size_t)row * H + 32 * nb + 4 * g;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float v[4];
          load4<T>(yrow + 8 * q, v);
          yv[4 * q] = v[0]; yv[4 * q + 1] = v[1]; yv[4 * q + 2] = v[2]; yv[4 * q + 3] = v[3];
        }
      }
      f32x16 d;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float v[4];
        load4<float>(dyrow + 32 * nb + 8 * q + 4 * g, v);
#pragma unroll
        for (int j = 0; j < 4; ++j) d[4 * q + j] = yv[4 * q + j] > 0.f ? v[j] : 0.f;
      }
      store_block_via_lds<T, H>((T *)a.dz2, row0, n_valid, nb, lane, d, stage);
#pragma unroll
      for (int q = 0; q < QB; ++q) dz2s[nb][q] = acc_slab<T>(d, q);
    }
  }

  // ---------------- dz1^T = (W2 dz2^T) * [z1^T > 0]: one group of W2^T fragments per block mb
  vec dz1s[MB][QB];
  {
    const vec *W2b = (const vec *)a.W2bt + lane;
    wg.begin(W2b, [&](int j) { return j * MB; }, GF);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      if (mb + 1 < MB) wg.fetch(W2b, [&](int j) { return j * MB + mb + 1; }, GF);
      f32x16 d;
#pragma unroll
      for (int r = 0; r < 16; ++r) d[r] = 0.f;
#pragma unroll
      for (int nb = 0; nb < MB; ++nb)
#pragma unroll
        for (int q = 0; q < QB; ++q)
          Opd::mma(wg.get(W2b, [&](int j) { return j * MB + mb; }, nb * QB + q), dz2s[nb][q], d);
      wg.next(mb + 1 < MB);
#pragma unroll
      for (int r = 0; r < 16; ++r) d[r] = acc1[mb][r] > 0.f ? d[r] : 0.f;
      store_block_via_lds<T, H>((T *)a.dz1, row0, n_valid, mb, lane, d, stage);
#pragma unroll
      for (int q = 0; q < QB; ++q) dz1s[mb][q] = acc_slab<T>(d, q);
    }
  }

  // ---------------- dx^T = W1 dz1^T over the first 2H input columns (h parts only): one group
  // of W1^T fragments per 32-column block kb of [part a | part b]
  if constexpr (KIND != KIND_EMBED) {
    const vec *W1b = (const vec *)a.W1bt + lane;
    constexpr int KB = 2 * MB;
    wg.begin(W1b, [&](int j) { return j * KB; }, GF);
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
      if (kb + 1 < KB) wg.fetch(W1b, [&](int j) { return j * KB + kb + 1; }, GF);
      f32x16 d;
#pragma unroll
      for (int r = 0; r < 16; ++r) d[r] = 0.f;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int q = 0; q < QB; ++q)
          Opd::mma(wg.get(W1b, [&](int j) { return j * KB + kb; }, mb * QB + q), dz1s[mb][q], d);
      wg.next(kb + 1 < KB);
      if constexpr (KIND == KIND_EDGE) {
        T *o = (T *)(kb < MB ? a.dx_a : a.dx_b);
        store_block_via_lds<T, H>(o, row0, n_valid, kb % MB, lane, d, stage);
      } else {
        float *o = (float *)(kb < MB ? a.dx_a : a.dx_b);
        store_block_via_lds<float, H>(o, row0, n_valid, kb % MB, lane, d, stage);
      }
    }
  }
}
