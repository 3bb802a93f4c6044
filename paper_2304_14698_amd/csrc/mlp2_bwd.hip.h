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

template <typename T1, typename T, int H, int KIND>
__global__ __launch_bounds__(256) void mlp2_bwd_kernel(const Mlp2BwdArgs a) {
  using Opd = Operand<T>;
  using vec = typename Opd::vec;
  constexpr int V = Opd::V, SL = 2 * V, MB = H / 32, HS = H / SL, QB = 32 / SL;
  using Opd1 = Operand<T1>;
  using vec1 = typename Opd1::vec;
  constexpr int V1 = Opd1::V, SL1 = 2 * V1;

  const int64_t per_xcd = (a.n_blocks + 7) / 8;
  const int64_t tile = (int64_t)(blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (tile >= a.n_blocks) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, g = lane >> 5;
  const int64_t row0 = (tile * 4 + wave) * 32;
  int64_t row = row0 + l32;
  const bool valid = row < a.n_rows;
  if (!valid) row = a.n_rows - 1;
  // every [rows, H] result leaves through a per-wave staging buffer, one 32-feature block at a time
  __shared__ __align__(16) char stage_all[4][BlockStage<float>::BYTES];
  char *stage = stage_all[wave];
  const int64_t left = a.n_rows - row0;
  const int n_valid = left < 32 ? (left > 0 ? (int)left : 0) : 32;

  // ---------------- z1^T = relu(W1^T x^T + b1), exactly as in the forward kernel
  f32x16 acc1[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc1[mb][r] = a.b1[32 * mb + acc_row(r, g)];
  const vec1 *W1 = (const vec1 *)a.W1s + lane;
  int64_t src = 0, dst = 0;
  if constexpr (KIND == KIND_EDGE) {
    src = a.in_src[row];
    dst = a.in_dst[row];
    const T *hs = (const T *)a.h + (size_t)src * H + g * V;
    const T *hd = (const T *)a.h + (size_t)dst * H + g * V;
#pragma unroll 2
    for (int s = 0; s < HS; ++s) {
      vec x = *(const vec *)(hs + s * SL);
      mma_slab<T, H>(W1 + (size_t)s * MB * 64, x, acc1);
    }
#pragma unroll 2
    for (int s = 0; s < HS; ++s) {
      vec x = *(const vec *)(hd + s * SL);
      mma_slab<T, H>(W1 + (size_t)(HS + s) * MB * 64, x, acc1);
    }
    const float *xe = a.edge_feat + (size_t)row * a.De;
    for (int s = 2 * HS; s < a.nslab1; ++s) {
      const vec x = tail_to_operand<T>(load_tail<V>(xe, a.De, s - 2 * HS, g));
      mma_slab<T, H>(W1 + (size_t)s * MB * 64, x, acc1);
    }
  } else if constexpr (KIND == KIND_NODE) {
    const T *hp = (const T *)a.h + (size_t)row * H + g * V;
    const T *ap = (const T *)a.agg + (size_t)row * H + g * V;
    const bool has_in = a.in_ptr[row + 1] > a.in_ptr[row];
#pragma unroll 2
    for (int s = 0; s < HS; ++s) {
      vec x = *(const vec *)(hp + s * SL);
      mma_slab<T, H>(W1 + (size_t)s * MB * 64, x, acc1);
    }
#pragma unroll 2
    for (int s = 0; s < HS; ++s) {
      vec x = has_in ? *(const vec *)(ap + s * SL) : Opd::zero();
      mma_slab<T, H>(W1 + (size_t)(HS + s) * MB * 64, x, acc1);
    }
  } else {
    const float *dn = a.node_dense + (size_t)row * a.Dd;
    const int op = a.node_op[row];
    const int e0 = a.in_ptr[row], e1 = a.in_ptr[row + 1];
    for (int s = 0; s < a.nslab1; ++s) {
      float a0[V1];
#pragma unroll
      for (int j = 0; j < V1; ++j) a0[j] = 0.f;
      if (s * SL1 + g * V1 < a.De)
        for (int e = e0; e < e1; ++e) {
          const float *xe = a.edge_feat + (size_t)e * a.De + s * SL1 + g * V1;
#pragma unroll
          for (int j = 0; j < V1; ++j)
            if (s * SL1 + g * V1 + j < a.De) a0[j] += xe[j];
        }
      vec1 x;
#pragma unroll
      for (int j = 0; j < V1; ++j) {
        const int k = s * SL1 + g * V1 + j;
        float v = 0.f;
        if (k < a.De) v = a0[j];
        else if (k < a.De + a.Tn) v = (k - a.De == op) ? 1.f : 0.f;
        else if (k < a.De + a.Tn + a.Dd) v = dn[k - a.De - a.Tn];
        x[j] = Opd1::from_float(v);
      }
      mma_slab<T1, H>(W1 + (size_t)s * MB * 64, x, acc1);
    }
  }
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
    for (int r = 0; r < 16; ++r) acc1[mb][r] = fmaxf(acc1[mb][r], 0.f);
    store_block_via_lds<T, H>((T *)a.z1, row0, n_valid, mb, lane, acc1[mb], stage);
  }

  // ---------------- dz2^T = dy^T * [y^T > 0], stored and kept as operand slabs
  vec dz2s[MB][QB];
  {
    const float *dyrow = a.dy + (size_t)(KIND == KIND_EDGE ? dst : row) * H;
    [[maybe_unused]] const vec *W2 = (const vec *)a.W2s + lane;
#pragma unroll
    for (int nb = 0; nb < MB; ++nb) {
      f32x16 yv;
      if constexpr (KIND == KIND_EDGE) {
#pragma unroll
        for (int r = 0; r < 16; ++r) yv[r] = a.b2[32 * nb + acc_row(r, g)];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
          for (int q = 0; q < QB; ++q) {
            vec z = acc_slab<T>(acc1[mb], q);
            vec w = W2[((size_t)(mb * QB + q) * MB + nb) * 64];
            Opd::mma(w, z, yv);
          }
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

  // ---------------- dz1^T = (W2 dz2^T) * [z1^T > 0]
  vec dz1s[MB][QB];
  {
    const vec *W2b = (const vec *)a.W2bt + lane;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      f32x16 d;
#pragma unroll
      for (int r = 0; r < 16; ++r) d[r] = 0.f;
#pragma unroll
      for (int nb = 0; nb < MB; ++nb)
#pragma unroll
        for (int q = 0; q < QB; ++q) {
          vec w = W2b[((size_t)(nb * QB + q) * MB + mb) * 64];
          Opd::mma(w, dz2s[nb][q], d);
        }
#pragma unroll
      for (int r = 0; r < 16; ++r) d[r] = acc1[mb][r] > 0.f ? d[r] : 0.f;
      store_block_via_lds<T, H>((T *)a.dz1, row0, n_valid, mb, lane, d, stage);
#pragma unroll
      for (int q = 0; q < QB; ++q) dz1s[mb][q] = acc_slab<T>(d, q);
    }
  }

  // ---------------- dx^T = W1 dz1^T over the first 2H input columns (h parts only)
  if constexpr (KIND != KIND_EMBED) {
    const vec *W1b = (const vec *)a.W1bt + lane;
    constexpr int KB = 2 * MB;                               // 32-column blocks of [part a | part b]
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
      f32x16 d;
#pragma unroll
      for (int r = 0; r < 16; ++r) d[r] = 0.f;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int q = 0; q < QB; ++q) {
          vec w = W1b[((size_t)(mb * QB + q) * KB + kb) * 64];
          Opd::mma(w, dz1s[mb][q], d);
        }
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
