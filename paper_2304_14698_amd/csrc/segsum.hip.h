// Deterministic segment sum over consecutive rows: out[s, :] = sum of rows [ptr[s], ptr[s+1]).
// Used for the receiver-side sum of incoming edge attributes (node-update layer, Section 3.4),
// the per-graph sum of node states (global-update layer); the backward pass gathers per node
// instead (node_grad_gather_kernel at the end of this file).
//
// Rows are cut into fixed sub-tiles of RT rows; D / VEC lanes own one sub-tile, each lane a
// 16-byte column slice. A lane walks its sub-tile in row order, so every sum has a fixed order
// (no atomics). A segment lying entirely inside a sub-tile is written directly; the piece of a
// segment that started in an earlier sub-tile goes to carry[st][0], the piece of one that
// continues into a later sub-tile to carry[st][1]; segsum_fixup adds the pieces in row order.
#pragma once
#include "mma.hip.h"

template <typename T, int VEC>
struct RowVec;
template <>
struct RowVec<float, 4> {
  static __device__ __forceinline__ void load(const float *p, float *v) {
    f32x4 x = *(const f32x4 *)p;
    v[0] = x[0]; v[1] = x[1]; v[2] = x[2]; v[3] = x[3];
  }
};
template <>
struct RowVec<bf16_t, 8> {
  static __device__ __forceinline__ void load(const bf16_t *p, float *v) {
    bf16x8 x = *(const bf16x8 *)p;
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = (float)x[j];
  }
};

template <typename TO>
__device__ __forceinline__ void store_out(TO *p, float v);
template <>
__device__ __forceinline__ void store_out<float>(float *p, float v) { *p = v; }
template <>
__device__ __forceinline__ void store_out<bf16_t>(bf16_t *p, float v) { *p = (bf16_t)v; }

// Output policy of the segment-sum kernels: plain store (empty segments get zeros).
struct PutStore {
  template <typename TO>
  static __device__ __forceinline__ void put(TO *p, float v) { store_out<TO>(p, v); }
  static constexpr bool kZeroEmpty = true;
};

// largest s in [0, n_seg) with ptr[s] <= row < ptr[s+1]; requires 0 <= row < ptr[n_seg]
__device__ __forceinline__ int seg_of_row(const int32_t *ptr, int64_t n_seg, int64_t row) {
  int64_t lo = 0, hi = n_seg;  // invariant: ptr[lo] <= row < ptr[hi]
  while (hi - lo > 1) {
    int64_t mid = (lo + hi) >> 1;
    if (ptr[mid] <= row) lo = mid; else hi = mid;
  }
  return (int)lo;
}

struct SegsumArgs {
  const void *vals;     // [*, D] rows, type TIn
  const int32_t *perm;  // nullable: row r of the reduction reads vals row perm[r]
  const int32_t *ptr;   // [n_seg + 1]
  const int32_t *row_seg;  // nullable: segment of vals row i (saves the search for a sub-tile's first segment)
  int64_t n_rows, n_seg;
  int D, RT;
  void *out;            // [n_seg, D], type TOut
  float *carry;         // [n_subtiles, 2, D]
};

template <typename TIn, typename TOut, int VEC, int RT, typename Put = PutStore>
__global__ __launch_bounds__(256) void segsum_kernel(const SegsumArgs a) {
  const int lpr = a.D / VEC;                                   // lanes per row
  const int64_t gt = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t st = gt / lpr;
  const int c = (int)(gt - st * lpr) * VEC;
  const int64_t r0 = st * RT;
  if (r0 >= a.n_rows) return;
  const int nv = (int)((a.n_rows - r0) < RT ? (a.n_rows - r0) : RT);
  const TIn *vals = (const TIn *)a.vals;
  TOut *out = (TOut *)a.out;
  float v[RT][VEC];
#pragma unroll
  for (int i = 0; i < RT; ++i) {
    if (i < nv) {
      int64_t r = a.perm ? (int64_t)a.perm[r0 + i] : (r0 + i);
      RowVec<TIn, VEC>::load(vals + (size_t)r * a.D + c, v[i]);
    }
  }
  int seg = a.row_seg ? a.row_seg[a.perm ? (int64_t)a.perm[r0] : r0] : seg_of_row(a.ptr, a.n_seg, r0);
  if (Put::kZeroEmpty && st == 0)                               // empty segments before row 0
    for (int s = 0; s < seg; ++s)
#pragma unroll
      for (int j = 0; j < VEC; ++j) store_out<TOut>(out + (size_t)s * a.D + c + j, 0.f);
  float acc[VEC];
#pragma unroll
  for (int j = 0; j < VEC; ++j) acc[j] = 0.f;
  bool first = true;
  int64_t seg_end = a.ptr[seg + 1];
#pragma unroll
  for (int i = 0; i < RT; ++i) {
    if (i < nv) {
      const int64_t row = r0 + i;
      while (row >= seg_end) {                                  // close finished (or empty) segments
        if (first && (int64_t)a.ptr[seg] < r0) {
#pragma unroll
          for (int j = 0; j < VEC; ++j) a.carry[((size_t)st * 2) * a.D + c + j] = acc[j];
        } else if (Put::kZeroEmpty || (int64_t)a.ptr[seg] < seg_end) {
#pragma unroll
          for (int j = 0; j < VEC; ++j) Put::put(out + (size_t)seg * a.D + c + j, acc[j]);
        }
        first = false;
#pragma unroll
        for (int j = 0; j < VEC; ++j) acc[j] = 0.f;
        ++seg;
        seg_end = a.ptr[seg + 1];
      }
#pragma unroll
      for (int j = 0; j < VEC; ++j) acc[j] += v[i][j];
    }
  }
  // last open segment of the sub-tile
  const int64_t tile_end = r0 + RT;                              // exclusive end of a full sub-tile
  if (first && (int64_t)a.ptr[seg] < r0) {
#pragma unroll
    for (int j = 0; j < VEC; ++j) a.carry[((size_t)st * 2) * a.D + c + j] = acc[j];
  } else if (seg_end > tile_end) {
#pragma unroll
    for (int j = 0; j < VEC; ++j) a.carry[((size_t)st * 2 + 1) * a.D + c + j] = acc[j];
  } else {
#pragma unroll
    for (int j = 0; j < VEC; ++j) Put::put(out + (size_t)seg * a.D + c + j, acc[j]);
  }
  // empty segments sitting exactly at this sub-tile's end (incl. trailing ones at n_rows)
  const int64_t here = r0 + nv;
  if (Put::kZeroEmpty && seg_end == here) {
    int s = seg + 1;
    while (s < a.n_seg && (int64_t)a.ptr[s + 1] == here) {
#pragma unroll
      for (int j = 0; j < VEC; ++j) store_out<TOut>(out + (size_t)s * a.D + c + j, 0.f);
      ++s;
    }
  }
}

// One thread per (sub-tile, 4-column slice): if the sub-tile's last segment starts inside it and
// runs on into later sub-tiles, add that segment's pieces in row order and write its sum.
// Loads are issued eight sub-tiles at a time; the additions keep the row order. row_seg
// (nullable) gives the segment of each row directly; otherwise it is found by binary search.
template <typename TOut, typename Put = PutStore>
__global__ __launch_bounds__(256) void segsum_fixup(const int32_t *ptr, const int32_t *row_seg,
                                                    int64_t n_rows, int64_t n_seg, int D, int RT,
                                                    const float *carry, TOut *out) {
  const int cpr = D / 4;                                        // column slices per sub-tile
  const int64_t gt = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t st = gt / cpr;
  const int c = (int)(gt - st * cpr) * 4;
  const int64_t r0 = st * RT;
  if (r0 >= n_rows) return;
  const int64_t nv = (n_rows - r0) < RT ? (n_rows - r0) : RT;
  const int64_t last = r0 + nv - 1;
  const int seg = row_seg ? row_seg[last] : seg_of_row(ptr, n_seg, last);
  const int64_t beg = ptr[seg], end = ptr[seg + 1];
  if (beg < r0 || end <= r0 + RT) return;
  f32x4 sum = *(const f32x4 *)(carry + ((size_t)st * 2 + 1) * D + c);
  const int64_t t_end = (end + RT - 1) / RT;                    // first sub-tile past the segment
  int64_t t = st + 1;
  for (; t + 8 <= t_end; t += 8) {
    f32x4 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = *(const f32x4 *)(carry + ((size_t)(t + i) * 2) * D + c);
#pragma unroll
    for (int i = 0; i < 8; ++i) sum += v[i];
  }
  for (; t < t_end; ++t) sum += *(const f32x4 *)(carry + ((size_t)t * 2) * D + c);
#pragma unroll
  for (int j = 0; j < 4; ++j) Put::put(out + (size_t)seg * D + c + j, sum[j]);
}

// The same fix-up for the message kernels' edge tiles, whose boundaries come from the packer's
// tile table: one thread per (tile, 4-column slice). Only receivers with more than 32 in-edges are
// ever cut by a tile boundary, so this kernel is launched only for batches that have one.
template <typename TOut>
__global__ __launch_bounds__(256) void edge_tile_fixup(const int32_t *tile_ptr, int64_t n_tiles,
                                                       const int32_t *in_ptr, const int32_t *in_dst, int D,
                                                       const float *carry, TOut *out) {
  const int cpr = D / 4;
  const int64_t gt = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t st = gt / cpr;
  const int c = (int)(gt - st * cpr) * 4;
  if (st >= n_tiles) return;
  const int64_t r0 = tile_ptr[st], r1 = tile_ptr[st + 1];
  const int seg = in_dst[r1 - 1];
  const int64_t beg = in_ptr[seg], end = in_ptr[seg + 1];
  if (beg < r0 || end <= r1) return;
  f32x4 sum = *(const f32x4 *)(carry + ((size_t)st * 2 + 1) * D + c);
  for (int64_t t = st + 1; t < n_tiles && tile_ptr[t] < end; ++t)
    sum += *(const f32x4 *)(carry + ((size_t)t * 2) * D + c);
#pragma unroll
  for (int j = 0; j < 4; ++j) store_out<TOut>(out + (size_t)seg * D + c + j, sum[j]);
}

// Backward of the message gathers, per node: dh[n] += sum over n's in-edges e of d_recv[e] + sum
// over n's out-edges (edge ids out_pos[k], k in [out_ptr[n], out_ptr[n+1])) of d_send[e]. One
// group of D / VEC lanes per node, each lane a 16-byte column slice; the edges are taken in index
// order and summed in fp32, so the result is run-to-run identical. One pass over dh instead of
// one per direction. recv_summed: d_recv is [n_nodes, D], already summed per receiver (rows of nodes
// without in-edges hold nothing and are not read).
// masked_out (or nullptr: the sum replaces dh): the sum goes there instead, multiplied by the ReLU
// mask of the layer that produced h -- ymask, the mask bits a forward kernel kept for its output
// (see Mlp2Args: [tiles of 32 nodes][D / 32][64 lanes] words; VEC must be 8) -- which is the dz2 the
// backward through that layer starts from.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void node_grad_gather_kernel(const T *d_recv, const T *d_send,
                                                               const int32_t *in_ptr, const int32_t *out_ptr,
                                                               const int32_t *out_pos, int64_t n_nodes, int D,
                                                               T *dh, int recv_summed, T *masked_out = nullptr,
                                                               const uint16_t *ymask = nullptr) {
  const int lpr = D / VEC;
  const int64_t gt = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t n = gt / lpr;
  if (n >= n_nodes) return;
  const int c = (int)(gt - n * lpr) * VEC;
  const int e0 = in_ptr[n], e1 = in_ptr[n + 1], k0 = out_ptr[n], k1 = out_ptr[n + 1];
  T *o = dh + (size_t)n * D + c;
  float acc[VEC], v[VEC];
  RowVec<T, VEC>::load(o, acc);
  if (recv_summed) {
    if (e1 > e0) {
      RowVec<T, VEC>::load(d_recv + (size_t)n * D + c, v);
#pragma unroll
      for (int j = 0; j < VEC; ++j) acc[j] += v[j];
    }
  } else {
    for (int e = e0; e < e1; ++e) {
      RowVec<T, VEC>::load(d_recv + (size_t)e * D + c, v);
#pragma unroll
      for (int j = 0; j < VEC; ++j) acc[j] += v[j];
    }
  }
  for (int k = k0; k < k1; ++k) {
    RowVec<T, VEC>::load(d_send + (size_t)out_pos[k] * D + c, v);
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc[j] += v[j];
  }
  if constexpr (VEC == 8) {
    if (masked_out) {
      // features c .. c+3 are accumulator registers 4 (c % 32 / 8) .. +3 of lane n % 32 of the node's
      // tile and feature block, features c+4 .. c+7 the same registers of lane n % 32 + 32
      const size_t w = ((size_t)(n / 32) * (D / 32) + c / 32) * 64 + (size_t)(n % 32);
      const unsigned lo = ymask[w] >> (4 * (c % 32 / 8)), hi = ymask[w + 32] >> (4 * (c % 32 / 8));
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        acc[j] = (lo >> j) & 1u ? acc[j] : 0.f;
        acc[4 + j] = (hi >> j) & 1u ? acc[4 + j] : 0.f;
      }
      o = masked_out + (size_t)n * D + c;
    }
  }
#pragma unroll
  for (int q = 0; q < VEC / 4; ++q) store4<T>(o + 4 * q, acc + 4 * q);
}
