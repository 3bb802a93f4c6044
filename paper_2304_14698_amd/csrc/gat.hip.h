// The graph-attention reading of the message-passing layer (second equation of Section 3.4, which
// cites graph attention for its learned per-edge weighting): per round
//   z = h W;  per edge j -> i: s = LeakyReLU_0.2(a_src . z_j + a_dst . z_i), likewise for a self
//   edge; alpha = softmax of s over i's in-edges plus the self edge;  h'_i = ReLU(sum alpha z_j).
// Two kernels: the dense part on the matrix cores (z and the two per-node scalars a_src . z,
// a_dst . z, taken from the fp32 accumulators), then a gather-bound pass over each receiver's
// contiguous in-edge range. The backward pass (further down) is gather-based as well: one
// pass per receiver for the softmax and score gradients, one per sender for dz, then two dense
// products (dh = dz W^T, dW = h^T dz) on the matrix cores.
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
  if (a.s_src && g == 0 && row0 + l32 < a.n_rows) {          // (null for the backward's dh = dz W^T)
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

// ---------------------------------------------------------------------------------------------
// Backward of the attention round. With dpre = dh' * [h' > 0] and, per receiver i, the softmax
// weights alpha over its in-edges k (sender j_k) and its self edge:
//   d alpha_k = dpre_i . z_{j_k},   sum_m alpha_m d alpha_m = dpre_i . pre_i = dpre_i . h'_i,
//   d u_k = alpha_k (d alpha_k - dpre_i . h'_i) * LeakyReLU'(u_k),   u_k = s_src[j_k] + s_dst[i],
//   dz_j = alpha_self,j dpre_j + sum over j's out-edges of alpha_k dpre_{i_k}
//          + a_src * (d u_self,j + sum over out-edges d u_k) + a_dst * (d u_self,j + sum over in-edges d u_k),
//   d a_src = sum_n d_ss[n] z_n,  d a_dst = sum_n d_sd[n] z_n,  dh = dz W^T,  dW = h^T dz.
struct GatBwdArgs {
  int64_t n_rows;
  const void *z, *hout, *dout;   // [N, H] operand type: saved z and h' of the round, upstream d h'
  const float *s_src, *s_dst;    // [N] saved scores
  const float *a_src, *a_dst;    // [H]
  const int32_t *in_ptr, *in_src, *in_dst, *out_ptr, *out_pos;
  float *alpha_e, *du_e;         // [E], receiver order
  float *alpha_s, *du_s;         // [N] self edge
  float *d_ss, *d_sd;            // [N] d / d s_src[n], d / d s_dst[n]
  void *dpre, *dz;               // [N, H] operand type
};

// sum over the `width` lanes of a lane group (width a power of two, groups aligned)
__device__ __forceinline__ float group_sum(float v, int width) {
  for (int o = width >> 1; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// Per receiver (a group of H / VEC lanes, each a 16-byte column slice): dpre, the softmax weights
// of its in-edges and self edge, and the gradients of their scores. Edges in order.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void gat_bwd_scores_kernel(const GatBwdArgs a, int H) {
  const int lpr = H / VEC;
  const int64_t gt = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t n = gt / lpr;
  const bool live = n < a.n_rows;                      // (whole groups; idle groups follow along for the shuffles)
  if (!live) n = a.n_rows - 1;
  const int c = (int)(gt % lpr) * VEC;
  const T *z = (const T *)a.z;
  float dp[VEC], hv[VEC], v[VEC];
  RowVec<T, VEC>::load((const T *)a.dout + (size_t)n * H + c, dp);
  RowVec<T, VEC>::load((const T *)a.hout + (size_t)n * H + c, hv);
  float ci = 0.f;
#pragma unroll
  for (int j = 0; j < VEC; ++j) {
    dp[j] = hv[j] > 0.f ? dp[j] : 0.f;
    ci = fmaf(dp[j], hv[j], ci);
  }
  ci = group_sum(ci, lpr);
  if (live) {
#pragma unroll
    for (int q = 0; q < VEC / 4; ++q) store4<T>((T *)a.dpre + (size_t)n * H + c + 4 * q, dp + 4 * q);
  }
  const int e0 = a.in_ptr[n], e1 = a.in_ptr[n + 1];
  const float sd = a.s_dst[n];
  const float u_self = a.s_src[n] + sd, s_self = leaky02(u_self);
  float mx = s_self;
  for (int e = e0; e < e1; ++e) mx = fmaxf(mx, leaky02(a.s_src[a.in_src[e]] + sd));
  float den = expf(s_self - mx);
  for (int e = e0; e < e1; ++e) den += expf(leaky02(a.s_src[a.in_src[e]] + sd) - mx);
  const float inv = 1.f / den;
  // self edge
  RowVec<T, VEC>::load(z + (size_t)n * H + c, v);
  float da = 0.f;
#pragma unroll
  for (int j = 0; j < VEC; ++j) da = fmaf(dp[j], v[j], da);
  da = group_sum(da, lpr);
  const float al_s = expf(s_self - mx) * inv;
  const float du_s = al_s * (da - ci) * (u_self > 0.f ? 1.f : 0.2f);
  float dsd = du_s;
  for (int e = e0; e < e1; ++e) {
    const int s = a.in_src[e];
    const float u = a.s_src[s] + sd;
    RowVec<T, VEC>::load(z + (size_t)s * H + c, v);
    float d = 0.f;
#pragma unroll
    for (int j = 0; j < VEC; ++j) d = fmaf(dp[j], v[j], d);
    d = group_sum(d, lpr);
    const float al = expf(leaky02(u) - mx) * inv;
    const float du = al * (d - ci) * (u > 0.f ? 1.f : 0.2f);
    dsd += du;
    if (live && c == 0) { a.alpha_e[e] = al; a.du_e[e] = du; }
  }
  if (live && c == 0) { a.alpha_s[n] = al_s; a.du_s[n] = du_s; a.d_sd[n] = dsd; }
}

// Per sender j (a group of H / VEC lanes): dz_j from its self edge, its out-edges (receiver-order
// positions out_pos[k], ascending) and the two score gradients; also d_ss[j].
template <typename T, int VEC>
__global__ __launch_bounds__(256) void gat_bwd_dz_kernel(const GatBwdArgs a, int H) {
  const int lpr = H / VEC;
  const int64_t gt = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t n = gt / lpr;
  if (n >= a.n_rows) return;
  const int c = (int)(gt - n * lpr) * VEC;
  const T *dpre = (const T *)a.dpre;
  float acc[VEC], v[VEC];
  RowVec<T, VEC>::load(dpre + (size_t)n * H + c, v);
  const float al_s = a.alpha_s[n];
#pragma unroll
  for (int j = 0; j < VEC; ++j) acc[j] = al_s * v[j];
  float dss = a.du_s[n];
  const int k0 = a.out_ptr[n], k1 = a.out_ptr[n + 1];
  for (int k = k0; k < k1; ++k) {
    const int e = a.out_pos[k];
    const float al = a.alpha_e[e];
    dss += a.du_e[e];
    RowVec<T, VEC>::load(dpre + (size_t)a.in_dst[e] * H + c, v);
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc[j] = fmaf(al, v[j], acc[j]);
  }
  const float dsd = a.d_sd[n];
#pragma unroll
  for (int j = 0; j < VEC; ++j) acc[j] += dss * a.a_src[c + j] + dsd * a.a_dst[c + j];
#pragma unroll
  for (int q = 0; q < VEC / 4; ++q) store4<T>((T *)a.dz + (size_t)n * H + c + 4 * q, acc + 4 * q);
  if (c == 0) a.d_ss[n] = dss;
}

// Partial sums of d a_src = sum_n d_ss[n] z_n and d a_dst = sum_n d_sd[n] z_n over a chunk of rows
// per block: partial[chunk][2][H]. Threads = H / VEC column slices x 256 / (H / VEC) row groups;
// a group walks its rows in order and the groups are added in group order (fixed order).
template <typename T, int VEC>
__global__ __launch_bounds__(256) void gat_avec_grad_kernel(const T *z, const float *d_ss, const float *d_sd,
                                                            int64_t n_rows, int rows_per_chunk, int H,
                                                            float *partial) {
  extern __shared__ __align__(16) float sm[];               // [groups][2][H]
  const int lpr = H / VEC, ng = 256 / lpr, t = threadIdx.x, c = (t % lpr) * VEC, q = t / lpr;
  const int64_t r0 = (int64_t)blockIdx.x * rows_per_chunk;
  int64_t r1 = r0 + rows_per_chunk;
  if (r1 > n_rows) r1 = n_rows;
  float as[VEC], ad[VEC], v[VEC];
#pragma unroll
  for (int j = 0; j < VEC; ++j) { as[j] = 0.f; ad[j] = 0.f; }
  for (int64_t r = r0 + q; r < r1; r += ng) {
    RowVec<T, VEC>::load(z + (size_t)r * H + c, v);
    const float ws = d_ss[r], wd = d_sd[r];
#pragma unroll
    for (int j = 0; j < VEC; ++j) { as[j] = fmaf(ws, v[j], as[j]); ad[j] = fmaf(wd, v[j], ad[j]); }
  }
#pragma unroll
  for (int j = 0; j < VEC; ++j) { sm[(q * 2) * H + c + j] = as[j]; sm[(q * 2 + 1) * H + c + j] = ad[j]; }
  __syncthreads();
  for (int i = t; i < 2 * H; i += 256) {
    float s = sm[i];
    for (int k = 1; k < ng; ++k) s += sm[(size_t)k * 2 * H + i];
    partial[(size_t)blockIdx.x * 2 * H + i] = s;
  }
}
