// Weight gradients of one affine layer, dW = X^T dZ and db = 1^T dZ, over a very tall X
// (rows = edges or nodes), deterministic: the rows are cut into chunks, every (column tile,
// chunk) block accumulates its partial [64, H] tile on the matrix cores in fp32, and a second
// kernel adds the chunk partials in chunk order onto the caller's gradient vector.
//
// The contraction runs over rows, so both MFMA operands need "lane = column, elements = rows".
// Row-major tiles are therefore transposed on their way into LDS: element (row, col) of a tile
// of TC columns lives at ((row / V) * TC' + col + col / V) * V + row % V (one pad column after
// every V keeps the transposing writes free of bank conflicts), which makes a lane's V rows of
// one column one 16-byte LDS read. The bias gradient comes from an extra all-ones column of X.
#pragma once
#include "mlp2.hip.h"

enum { WG_PLAIN = 0, WG_EDGE = 1, WG_NODE = 2, WG_EMBED = 3 };

struct WgradArgs {
  int64_t n_rows;
  int rows_per_chunk, n_chunks;
  int Ka;                   // real columns of X; column Ka is the all-ones bias column
  const void *A;            // PLAIN: [rows, Ka] operand type (Ka == H)
  const void *h, *agg;      // EDGE / NODE sources, operand type
  const int32_t *in_ptr, *in_src, *in_dst;
  const float *edge_feat;
  const int32_t *node_op;
  const float *node_dense;
  int De, Tn, Dd;
  const void *dZ;           // [rows, H] operand type
  float *partial;           // [n_chunks, KaP, H], KaP = 64 * gridDim.x
};

// V consecutive columns (col0 .. col0+V-1, col0 a multiple of V) of row `row` of the virtual X.
template <typename T, int H, int KIND>
__device__ __forceinline__ typename Operand<T>::vec wgrad_load_x(const WgradArgs &a, int64_t row,
                                                                 int col0) {
  using Opd = Operand<T>;
  constexpr int V = Opd::V;
  typename Opd::vec x;
  if constexpr (KIND == WG_PLAIN) {
    if (col0 + V <= a.Ka) return *(const typename Opd::vec *)((const T *)a.A + (size_t)row * a.Ka + col0);
#pragma unroll
    for (int j = 0; j < V; ++j) x[j] = Opd::from_float(col0 + j == a.Ka ? 1.f : 0.f);
    return x;
  } else if constexpr (KIND == WG_EDGE) {
    if (col0 + V <= H) return *(const typename Opd::vec *)((const T *)a.h + (size_t)a.in_src[row] * H + col0);
    if (col0 + V <= 2 * H)
      return *(const typename Opd::vec *)((const T *)a.h + (size_t)a.in_dst[row] * H + (col0 - H));
#pragma unroll
    for (int j = 0; j < V; ++j) {
      const int k = col0 + j - 2 * H;
      x[j] = Opd::from_float(k < a.De ? a.edge_feat[(size_t)row * a.De + k] : (k == a.De ? 1.f : 0.f));
    }
    return x;
  } else if constexpr (KIND == WG_NODE) {
    if (col0 + V <= H) return *(const typename Opd::vec *)((const T *)a.h + (size_t)row * H + col0);
    if (col0 + V <= 2 * H) {
      if (a.in_ptr[row + 1] > a.in_ptr[row])
        return *(const typename Opd::vec *)((const T *)a.agg + (size_t)row * H + (col0 - H));
      return Opd::zero();
    }
#pragma unroll
    for (int j = 0; j < V; ++j) x[j] = Opd::from_float(col0 + j == 2 * H ? 1.f : 0.f);
    return x;
  } else {
    const int op = a.node_op[row];
#pragma unroll
    for (int j = 0; j < V; ++j) {
      const int k = col0 + j;
      float v = 0.f;
      if (k < a.De) {
        for (int e = a.in_ptr[row]; e < a.in_ptr[row + 1]; ++e) v += a.edge_feat[(size_t)e * a.De + k];
      } else if (k < a.De + a.Tn) v = (k - a.De == op) ? 1.f : 0.f;
      else if (k < a.De + a.Tn + a.Dd) v = a.node_dense[(size_t)row * a.Dd + (k - a.De - a.Tn)];
      else if (k == a.De + a.Tn + a.Dd) v = 1.f;
      x[j] = Opd::from_float(v);
    }
    return x;
  }
}

template <typename T, int H, int KIND>
__global__ __launch_bounds__(256) void wgrad_kernel(const WgradArgs a) {
  using Opd = Operand<T>;
  using vec = typename Opd::vec;
  constexpr int V = Opd::V;            // rows per lane per MFMA step; a step covers 2V rows
  constexpr int TA = 64;               // X columns per block
  constexpr int RS = 8 * V;            // rows per stage (64 bf16, 32 fp32: LDS stays under 48 KB)
  constexpr int NB = H / 64;           // 32-column blocks of dZ per wave
  __shared__ T As[RS / V][TA + TA / V][V];
  __shared__ T Bs[RS / V][H + H / V][V];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, g = lane >> 5;
  const int ka0 = blockIdx.x * TA;
  const int chunk = blockIdx.y;
  const int64_t r_begin = (int64_t)chunk * a.rows_per_chunk;
  int64_t r_end = r_begin + a.rows_per_chunk;
  if (r_end > a.n_rows) r_end = a.n_rows;
  const int kab = wave & 1;            // this wave's 32-column block of X inside the tile
  const int kbb0 = wave >> 1;          // its dZ blocks: kbb0, kbb0 + 2, ...

  f32x16 acc[NB];
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

  for (int64_t rs = r_begin; rs < r_end; rs += RS) {
    // ---- stage X tile: RS rows x TA columns, V-column vectors; lanes run over column chunks
    for (int vi = tid; vi < RS * (TA / V); vi += 256) {
      const int cc = vi % (TA / V), rl = vi / (TA / V);
      const int64_t row = rs + rl;
      vec x = row < r_end ? wgrad_load_x<T, H, KIND>(a, row, ka0 + cc * V) : Opd::zero();
#pragma unroll
      for (int j = 0; j < V; ++j) As[rl / V][cc * (V + 1) + j][rl % V] = x[j];
    }
    for (int vi = tid; vi < RS * (H / V); vi += 256) {
      const int cc = vi % (H / V), rl = vi / (H / V);
      const int64_t row = rs + rl;
      vec x = row < r_end ? *(const vec *)((const T *)a.dZ + (size_t)row * H + cc * V) : Opd::zero();
#pragma unroll
      for (int j = 0; j < V; ++j) Bs[rl / V][cc * (V + 1) + j][rl % V] = x[j];
    }
    __syncthreads();
    // ---- contraction over the stage's rows, 2V rows per step
#pragma unroll
    for (int st = 0; st < RS / (2 * V); ++st) {
      const int ca = 32 * kab + l32;
      const vec xa = *(const vec *)&As[2 * st + g][ca + ca / V][0];
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int cb = 32 * (kbb0 + 2 * i) + l32;
        const vec xb = *(const vec *)&Bs[2 * st + g][cb + cb / V][0];
        Opd::mma(xa, xb, acc[i]);
      }
    }
    __syncthreads();
  }
  const int KaP = TA * gridDim.x;
  float *out = a.partial + ((size_t)chunk * KaP + ka0 + 32 * kab) * H;
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r)
      out[(size_t)acc_row(r, g) * H + 32 * (kbb0 + 2 * i) + l32] = acc[i][r];
}

// dW[k, f] += sum over chunks of partial[chunk, k, f] for k < Ka; db[f] += row Ka. A block handles
// 32 consecutive entries; its 8 thread groups take every eighth chunk (eight loads in flight
// each) and their sums are added in group order, so the result has one fixed summation order.
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float *partial, int n_chunks, int KaP, int Ka,
                                                           int H, float *dW, float *db) {
  __shared__ float part[8][32];
  const int e = threadIdx.x & 31, g = threadIdx.x >> 5;
  const int64_t i = (int64_t)blockIdx.x * 32 + e;
  const bool live = i < (int64_t)(Ka + 1) * H;
  const int k = live ? (int)(i / H) : 0, f = live ? (int)(i - (int64_t)k * H) : 0;
  const float *p = partial + (size_t)k * H + f;
  const size_t cs = (size_t)KaP * H;
  float s = 0.f;
  int c = g;
  for (; c + 56 < n_chunks; c += 64) {
    float v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = p[(size_t)(c + 8 * j) * cs];
#pragma unroll
    for (int j = 0; j < 8; ++j) s += v[j];
  }
  for (; c < n_chunks; c += 8) s += p[(size_t)c * cs];
  part[g][e] = s;
  __syncthreads();
  if (g == 0 && live) {
    float t = part[0][e];
#pragma unroll
    for (int j = 1; j < 8; ++j) t += part[j][e];
    if (k < Ka) dW[(size_t)k * H + f] += t;
    else db[f] += t;
  }
}
