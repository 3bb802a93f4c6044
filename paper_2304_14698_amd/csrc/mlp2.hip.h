// Fused two-layer ReLU MLP over a tile of rows, both layers on the matrix cores, the hidden
// activation never leaving registers. One kernel template serves the three learned transforms of
// the encoder (Section 3.4):
//   EMBED  rows = nodes,  x = [sum of incoming edge attrs | one-hot op | dense attrs]   -> h0
//          (the sum over the node's in-edges is formed in the prologue)
//   EDGE   rows = edges in receiver order, x = [h_sender | h_receiver | edge attrs]
//          -> ReLU MLP -> summed per receiver (the message-passing sum)                 -> agg
//   NODE   rows = nodes,  x = [h | agg]                                                 -> h'
//
// Each wave owns 32 rows. Layer 1 is computed transposed (features x rows: the weights are the
// A operand, the gathered input rows the B operand, loaded straight from global memory into
// registers), so its accumulator layout (lane = row, registers = features) is exactly the
// A-operand layout layer 2 needs; layer 2 then yields rows x features with lane = feature,
// registers = rows, which makes the per-receiver sum a walk down each lane's column.
// Weights are pre-arranged on the host in the per-lane fragment order (see swizzle_* in the
// runtime), so every weight fragment is one coalesced 1 KB load per wave.
#pragma once
#include "mma.hip.h"
#include "segsum.hip.h"

enum { KIND_EMBED = 0, KIND_EDGE = 1, KIND_NODE = 2 };

struct Mlp2Args {
  int64_t n_rows;
  int64_t n_blocks;        // number of 128-row tiles
  const void *W1s, *W2s;   // fragment-ordered weights, operand type
  const float *b1, *b2;    // [H]
  int nslab1;              // slabs of layer 1's (zero-padded) input width
  const void *h;           // [N, H] operand type            (EDGE, NODE)
  const void *agg;         // [N, H] operand type            (NODE)
  const int32_t *in_ptr;   // [N + 1]                        (all kinds)
  const int32_t *in_src;   // [E]                            (EDGE)
  const int32_t *in_dst;   // [E]                            (EDGE)
  const float *edge_feat;  // [E, De] receiver order         (EDGE, EMBED)
  const int32_t *node_op;  // [N]                            (EMBED)
  const float *node_dense; // [N, Dd]                        (EMBED)
  int De, Tn, Dd;
  void *out;               // [N, H] operand type
  float *carry;            // [ceil(E / 32), 2, H]           (EDGE)
};

template <typename T, int H>
__device__ __forceinline__ void mma_slab(const typename Operand<T>::vec *wp,
                                         const typename Operand<T>::vec &x, f32x16 *acc) {
#pragma unroll
  for (int mb = 0; mb < H / 32; ++mb) {
    typename Operand<T>::vec w = wp[mb * 64];
    Operand<T>::mma(w, x, acc[mb]);
  }
}

// T1 = operand type of layer 1 (its input rows and W1), T = operand type of layer 2 and of the
// stored activations. They differ only for EMBED in bf16 mode, whose first layer stays in fp32:
// its inputs (log2 shape attributes up to 12, sums of edge attributes) are large enough for bf16
// weight rounding to dominate the error of the whole encoder.
template <typename T1, typename T, int H, int KIND>
__global__ __launch_bounds__(256) void mlp2_kernel(const Mlp2Args a) {
  using Opd = Operand<T>;
  using vec = typename Opd::vec;
  constexpr int V = Opd::V, SL = 2 * V, MB = H / 32, HS = H / SL;
  using Opd1 = Operand<T1>;
  using vec1 = typename Opd1::vec;
  constexpr int V1 = Opd1::V, SL1 = 2 * V1;
  static_assert(KIND == KIND_EMBED || sizeof(T1) == sizeof(T), "only EMBED mixes operand types");
  __shared__ float zb[KIND == KIND_EDGE ? 4 : 1][32][64];

  // consecutive tiles stay on one XCD (blocks are dealt round-robin to the 8 XCDs), so the rows
  // a tile gathers are mostly in that XCD's L2 already
  const int64_t per_xcd = (a.n_blocks + 7) / 8;
  const int64_t tile = (int64_t)(blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (tile >= a.n_blocks) return;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, g = lane >> 5;
  const int64_t wt = tile * 4 + wave;                           // wave tile = 32 rows
  const int64_t row0 = wt * 32;
  int64_t row = row0 + l32;
  if (row >= a.n_rows) row = a.n_rows - 1;                      // clamp loads; stores are guarded

  // ---------------- layer 1: acc1[mb] = (W1^T x^T) tile, features x rows, bias pre-loaded
  f32x16 acc1[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc1[mb][r] = a.b1[32 * mb + acc_row(r, g)];
  const vec1 *W1 = (const vec1 *)a.W1s + lane;

  if constexpr (KIND == KIND_EDGE) {
    const T *hs = (const T *)a.h + (size_t)a.in_src[row] * H + g * V;
    const T *hd = (const T *)a.h + (size_t)a.in_dst[row] * H + g * V;
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
      vec x;
#pragma unroll
      for (int j = 0; j < V; ++j) {
        const int k = (s - 2 * HS) * SL + g * V + j;
        x[j] = Opd::from_float(k < a.De ? xe[k] : 0.f);
      }
      mma_slab<T, H>(W1 + (size_t)s * MB * 64, x, acc1);
    }
  } else if constexpr (KIND == KIND_NODE) {
    const T *hp = (const T *)a.h + (size_t)row * H + g * V;
    const T *ap = (const T *)a.agg + (size_t)row * H + g * V;
    const bool has_in = a.in_ptr[row + 1] > a.in_ptr[row];      // agg rows of source nodes are unwritten
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
    // the sum of the node's incoming edge attributes is formed here, from the node's contiguous
    // receiver-order edge range, in edge order
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

  // ---------------- layer 2: acc2[nb] = relu(z1) W2 tile, rows x features, bias pre-loaded
  f32x16 acc2[MB];
#pragma unroll
  for (int nb = 0; nb < MB; ++nb) {
    const float bv = a.b2[32 * nb + l32];
#pragma unroll
    for (int r = 0; r < 16; ++r) acc2[nb][r] = bv;
  }
  const vec *W2 = (const vec *)a.W2s + lane;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
    for (int q = 0; q < 32 / SL; ++q) {
      vec z;
#pragma unroll
      for (int j = 0; j < V; ++j) z[j] = Opd::from_float(fmaxf(acc1[mb][q * V + j], 0.f));
      const vec *wp = W2 + (size_t)(mb * (32 / SL) + q) * MB * 64;
#pragma unroll
      for (int nb = 0; nb < MB; ++nb) {
        vec w = wp[nb * 64];
        Opd::mma(z, w, acc2[nb]);
      }
    }
  }

  // ---------------- epilogue
  T *out = (T *)a.out;
  if constexpr (KIND != KIND_EDGE) {
#pragma unroll
    for (int nb = 0; nb < MB; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t rr = row0 + acc_row(r, g);
        if (rr < a.n_rows) out[(size_t)rr * H + 32 * nb + l32] = Opd::from_float(fmaxf(acc2[nb][r], 0.f));
      }
  } else {
    const int dstv = a.in_dst[row];
    const int64_t left = a.n_rows - row0;
    const int nv = left < 32 ? (int)left : 32;                  // <= 0 for a wave past the end
#pragma unroll
    for (int ch = 0; ch < H / 64; ++ch) {
#pragma unroll
      for (int nbl = 0; nbl < 2; ++nbl)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          zb[wave][acc_row(r, g)][32 * nbl + l32] = fmaxf(acc2[2 * ch + nbl][r], 0.f);
      __syncthreads();
      if (nv > 0) {
        const int f = 64 * ch + lane;
        float sum = 0.f;
        int prev = __builtin_amdgcn_readlane(dstv, 0);
        bool first = true;
        for (int i = 0; i < nv; ++i) {
          const int cur = __builtin_amdgcn_readlane(dstv, i);
          if (cur != prev) {                                    // receiver `prev` is finished
            if (first && (int64_t)a.in_ptr[prev] < row0) a.carry[((size_t)wt * 2) * H + f] = sum;
            else out[(size_t)prev * H + f] = Opd::from_float(sum);
            first = false;
            sum = 0.f;
            prev = cur;
          }
          sum += zb[wave][i][lane];
        }
        if (first && (int64_t)a.in_ptr[prev] < row0) a.carry[((size_t)wt * 2) * H + f] = sum;
        else if ((int64_t)a.in_ptr[prev + 1] > row0 + 32) a.carry[((size_t)wt * 2 + 1) * H + f] = sum;
        else out[(size_t)prev * H + f] = Opd::from_float(sum);
      }
      __syncthreads();
    }
  }
}
