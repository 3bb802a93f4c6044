// The graph-attention reading of the message-passing layer (second equation of Section 3.4, which
// cites graph attention for its learned per-edge weighting): per round
//   z = h W;  per edge j -> i: s = LeakyReLU_0.2(a_src . z_j + a_dst . z_i), likewise for a self
//   edge; alpha = softmax of s over i's in-edges plus the self edge;  h'_i = ReLU(sum alpha z_j).
// Two kernels: the dense part on the matrix cores (z and the two per-node scalars a_src . z,
// a_dst . z, taken from the fp32 accumulators), then a gather-bound pass over each receiver's
// contiguous in-edge range. Forward only.
#pragma once
#include "mlp2.hip.h"

struct GatArgs {
  int64_t n_rows, n_blocks;      // nodes; 128-row tiles
  const void *h;                 // [N, H] operand type
  const void *Ws;                // fragment-ordered W [H, H], operand type
  const float *a_src, *a_dst;    // [H]
  void *z;                       // [N, H] operand type
  float *s_src, *s_dst;          // [N]
  const int32_t *in_ptr, *in_src;
  void *out;                     // [N, H] operand type
};

// z = h W for a tile of 32 rows per wave (features x rows, as the fused MLP's first layer), the
// two attention scalars of each row from the accumulators, z stored as whole rows.
template <typename T, int H>
__global__ __launch_bounds__(256) void gat_linear_kernel(const GatArgs a) {
  using Opd = Operand<T>;
  using vec = typename Opd::vec;
  constexpr int V = Opd::V, SL = 2 * V, MB = H / 32, HS = H / SL;
  __shared__ __align__(16) char stage[4][RowStage<T, H>::BYTES];
  const int64_t per_xcd = (a.n_blocks + 7) / 8;
  const int64_t tile = (int64_t)(blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (tile >= a.n_blocks) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, g = lane >> 5;
  const int64_t row0 = (tile * 4 + wave) * 32;
  if (row0 >= a.n_rows) return;
  int64_t row = row0 + l32;
  if (row >= a.n_rows) row = a.n_rows - 1;
  f32x16 acc[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mb][r] = 0.f;
  const vec *W = (const vec *)a.Ws + lane;
  const T *hp = (const T *)a.h + (size_t)row * H + g * V;
  vec x[HS];
#pragma unroll
  for (int s = 0; s < HS; ++s) x[s] = *(const vec *)(hp + s * SL);
#pragma unroll
  for (int s = 0; s < HS; ++s) mma_slab<T, H>(W + (size_t)s * MB * 64, x[s], acc);
  float ps = 0.f, pd = 0.f;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const f32x4 as = *(const f32x4 *)(a.a_src + 32 * mb + 8 * q + 4 * g);
      const f32x4 ad = *(const f32x4 *)(a.a_dst + 32 * mb + 8 * q + 4 * g);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        ps = fmaf(acc[mb][4 * q + j], as[j], ps);
        pd = fmaf(acc[mb][4 * q + j], ad[j], pd);
      }
    }
  ps += __shfl_xor(ps, 32);                                     // the row's other half of the features
  pd += __shfl_xor(pd, 32);
  if (g == 0 && row0 + l32 < a.n_rows) {
    a.s_src[row] = ps;
    a.s_dst[row] = pd;
  }
  T *z = (T *)a.z;
  store_rows_via_lds<T, H, false>(acc, stage[wave], lane, [&](int r) -> T * {
    return row0 + r < a.n_rows ? z + (size_t)(row0 + r) * H : nullptr;
  });
}

__device__ __forceinline__ float leaky02(float x) { return x > 0.f ? x : 0.2f * x; }

// One receiver per group of H * sizeof(T) / 16 lanes, each lane a 16-byte column slice: softmax
// over the receiver's in-edges (contiguous in receiver order) plus the self edge, weighted sum
// of the gathered z rows, ReLU. Edges are taken in order, so the result is run-to-run identical.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void gat_aggregate_kernel(const GatArgs a, int H) {
  const int lpr = H / VEC;
  const int64_t gt = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t n = gt / lpr;
  if (n >= a.n_rows) return;
  const int c = (int)(gt - n * lpr) * VEC;
  const T *z = (const T *)a.z;
  const int e0 = a.in_ptr[n], e1 = a.in_ptr[n + 1];
  const float sd = a.s_dst[n];
  const float s_self = leaky02(a.s_src[n] + sd);
  float mx = s_self;
  for (int e = e0; e < e1; ++e) mx = fmaxf(mx, leaky02(a.s_src[a.in_src[e]] + sd));
  float den = expf(s_self - mx);
  float acc[VEC], v[VEC];
  RowVec<T, VEC>::load(z + (size_t)n * H + c, v);
#pragma unroll
  for (int j = 0; j < VEC; ++j) acc[j] = den * v[j];
  for (int e = e0; e < e1; ++e) {
    const int s = a.in_src[e];
    const float w = expf(leaky02(a.s_src[s] + sd) - mx);
    den += w;
    RowVec<T, VEC>::load(z + (size_t)s * H + c, v);
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc[j] = fmaf(w, v[j], acc[j]);
  }
  const float inv = 1.f / den;
  T *o = (T *)a.out + (size_t)n * H + c;
#pragma unroll
  for (int q = 0; q < VEC / 4; ++q) {
    float r[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) r[j] = fmaxf(acc[4 * q + j] * inv, 0.f);
    store4<T>(o + 4 * q, r);
  }
}
