// Fused two-layer ReLU MLP over a tile of rows, both layers on the matrix cores, the hidden
// activation never leaving registers. One kernel template serves the three learned transforms of
// the encoder (Section 3.4):
//   EMBED  rows = nodes,  x = [sum of incoming edge attrs | one-hot op | dense attrs]   -> h0
//          (the sum over the node's in-edges is formed in the prologue)
//   EDGE   rows = edges in receiver order, x = [h_sender | h_receiver | edge attrs]
//          -> ReLU MLP -> summed per receiver (the message-passing sum)                 -> agg
//   NODE   rows = nodes,  x = [h | agg]                                                 -> h'
//
// Each wave owns 32 rows. Both layers are computed transposed (features x rows: the weights are
// the A operand, the gathered input rows the B operand, loaded straight from global memory into
// registers), so layer 1's accumulator layout (lane = row, registers = features) is, after ReLU
// and conversion, the B-operand layout of layer 2; layer 2's accumulators have lane = row as
// well, so a row leaves as register quads and the per-receiver sum runs across adjacent lanes.
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
  const int32_t *agg_src;  // [N] NODE: the row of agg that holds a node's received sum, -1 for a node without
                           //   in-edges (the message kernels never write its row: zeros are read in its place);
                           //   nullptr: every node reads its own row
  const int32_t *in_ptr;   // [N + 1]                        (all kinds)
  const int32_t *in_src;   // [E]                            (EDGE)
  const int32_t *in_dst;   // [E]                            (EDGE)
  const float *edge_feat;  // [E, De] receiver order         (EDGE, EMBED)
  const int32_t *node_op;  // [N]                            (EMBED)
  const float *node_dense; // [N, Dd]                        (EMBED)
  int De, Tn, Dd;
  const void *W1x;         // EMBED: fragment-ordered fp32 rows of W1 for [edge-attr sum | dense attrs]
  int nslabx;              // EMBED: its slabs
  const float *table;      // EMBED: [Tn, H] fp32 rows of W1 for the one-hot op type
  const void *zero_row;    // 1 KB of zeros (source of rows that are absent)
  void *agg0;              // EMBED: first of n_agg received-sum buffers [N, H], agg_stride bytes apart;
  size_t agg_stride;       //        the embed kernel zeroes their rows of nodes without in-edges, which
  int n_agg;               //        the message kernels never write (0 when the readers go by agg_src)
  void *out;               // [N, H] operand type
  void *z1;                // kernels instantiated to keep the forward for the backward pass: the hidden
  uint16_t *z1mask;        //   activation relu(z1) [rows, H] operand type (an operand of the weight gradient)
  uint16_t *ymask;         //   and the ReLU masks of z1 and of y, which is all the backward through the MLP
                           //   needs of the forward: [tiles][H / 32][64 lanes] words, bit r of lane l =
                           //   accumulator register r of that lane (its row, its feature block) > 0. Tiles are
                           //   the kernel's wave tiles: edge tiles, or 32 consecutive nodes
  float *carry;            // [n_tiles, 2, H]                (EDGE)
  const int32_t *tile_ptr; // [n_tiles + 1] first edge of each edge tile (EDGE)
  int64_t n_tiles;         //                                (EDGE)
};

// Raw (fp32) piece of one row's trailing attributes that lane group g feeds to slab `ts` of the
// tail: columns [ts*2V + g*V, +V) of a row of `width` floats (width a multiple of 4), zeros
// beyond. The loads are unconditional (out-of-range pieces re-read the row's first columns and
// are zeroed afterwards) so that no branch or early wait separates them from other loads.
template <int V>
struct TailRaw {
  f32x4 q[V / 4];
};
// (the two halves -- request, then zeroing at the point of use -- are separate so that a caller
// can request a tile ahead without the zeroing's wait landing next to the request)
template <int V>
__device__ __forceinline__ TailRaw<V> request_tail(const float *rowp, int width, int ts, int g) {
  TailRaw<V> r;
#pragma unroll
  for (int i = 0; i < V / 4; ++i) {
    const int k = ts * 2 * V + g * V + 4 * i;
    r.q[i] = *(const f32x4 *)(rowp + (k + 4 <= width ? k : 0));
  }
  return r;
}
template <int V>
__device__ __forceinline__ TailRaw<V> zero_tail_beyond(TailRaw<V> r, int width, int ts, int g) {
#pragma unroll
  for (int i = 0; i < V / 4; ++i)
    if (ts * 2 * V + g * V + 4 * i + 4 > width) r.q[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  return r;
}
template <int V>
__device__ __forceinline__ TailRaw<V> load_tail(const float *rowp, int width, int ts, int g) {
  return zero_tail_beyond<V>(request_tail<V>(rowp, width, ts, g), width, ts, g);
}
template <typename T>
__device__ __forceinline__ typename Operand<T>::vec tail_to_operand(const TailRaw<Operand<T>::V> &r);
template <>
__device__ __forceinline__ f32x4 tail_to_operand<float>(const TailRaw<4> &r) { return r.q[0]; }
template <>
__device__ __forceinline__ bf16x8 tail_to_operand<bf16_t>(const TailRaw<8> &r) {
  return pack_bf16x8(r.q[0][0], r.q[0][1], r.q[0][2], r.q[0][3], r.q[1][0], r.q[1][1], r.q[1][2], r.q[1][3]);
}

template <typename T, int H>
__device__ __forceinline__ void mma_slab(const typename Operand<T>::vec *wp,
                                         const typename Operand<T>::vec &x, f32x16 *acc) {
#pragma unroll
  for (int mb = 0; mb < H / 32; ++mb) {
    typename Operand<T>::vec w = wp[mb * 64];
    Operand<T>::mma(w, x, acc[mb]);
  }
}

// Receivers of the edges of a wave tile (edges [e0, e0 + nv), nv <= 32, from the packer's tile
// table), plus those of the edges just outside it.
struct EdgeTileMeta {
  int dst;      // receiver of this lane's edge (lanes 32..63 mirror 0..31; lanes past the tile's
                // last edge repeat it)
  int prev_d;   // receiver of the edge before the tile, -1 if there is none
  int next_d;   // receiver of the edge after the tile, -1 if there is none
};
__device__ __forceinline__ EdgeTileMeta load_edge_meta(const int32_t *in_dst, int64_t n_rows, int64_t e0, int nv,
                                                       int l32) {
  EdgeTileMeta m;
  m.dst = in_dst[e0 + (l32 < nv ? l32 : nv - 1)];
  m.prev_d = e0 > 0 ? in_dst[e0 - 1] : -1;
  m.next_d = e0 + nv < n_rows ? in_dst[e0 + nv] : -1;
  return m;
}

// The mask bits (value > 0) of this lane's 16 registers of one accumulator block.
__device__ __forceinline__ uint16_t lane_mask_bits(const f32x16 &acc) {
  uint32_t m = 0;
#pragma unroll
  for (int r = 0; r < 16; ++r) m |= (acc[r] > 0.f ? 1u : 0u) << r;
  return (uint16_t)m;
}

// Per-receiver sum of a wave tile of messages held as features x rows accumulators (lane = edge,
// registers = features; edges are in receiver order, so a receiver's edges are adjacent lanes).
// ReLU, then a segmented suffix sum across lanes by doubling: after the step of distance d a lane
// holds the sum of its own and the next 2d - 1 edges of its receiver, so the first lane of every
// receiver ends with the receiver's total after ceil(log2(longest run)) steps (none at all when
// every receiver of the tile has one in-edge, one when none has more than two). The order of
// the additions is fixed by the positions in the tile alone. The total held by the first lane of
// each run then goes to out[receiver] (whole rows, through the staging buffer) when the run lies
// inside the tile, to
// carry[wt][0] when it began before the tile, to carry[wt][1] when it goes on after it (a run
// covering the whole tile and open on both sides counts as begun before); segsum_fixup adds the
// carried pieces in tile order.
template <typename T, int H>
__device__ __forceinline__ void edge_tile_sum(f32x16 (&acc)[H / 32], const EdgeTileMeta &m, int64_t wt, int nv,
                                               int lane, T *out, float *carry, char *stage) {
  constexpr int MB = H / 32;
  const int l32 = lane & 31, g = lane >> 5;
  const bool valid = l32 < nv;                                  // nv >= 1
  const int up = __shfl_up(m.dst, 1);                           // lane 32 reads lane 31, but is a head anyway
  const bool head = valid && (l32 == 0 || up != m.dst);
  const uint64_t heads = ((uint64_t)(uint32_t)__ballot(head)) | ((uint64_t)1 << nv);
  // number of edges after this one that have the same receiver and lie in the tile
  const int rem = valid ? __builtin_ctzll(heads >> (l32 + 1)) : 0;
#pragma unroll
  for (int nb = 0; nb < MB; ++nb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[nb][r] = relu_f32(acc[nb][r]);
  // (the lane's partner value enters through a product with 0 or 1: one fused multiply-add per
  // register instead of a select and an add; the values are finite sums of ReLU outputs)
  if (__any(rem >= 1)) {
    // first step, the only one for in-degrees up to 2: the neighbouring lane's value by a
    // wave-wide shift (no LDS traffic)
    const float takef = rem >= 1 ? 1.f : 0.f;
#pragma unroll
    for (int nb = 0; nb < MB; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        // (a copy first: bit-casting the vector-element lvalue itself reads element 0)
        const float v = acc[nb][r];
        const float t = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x130, 0xf, 0xf, false));
        acc[nb][r] = fmaf(t, takef, v);
      }
  }
  for (int d = 2; __any(rem >= d); d <<= 1) {
    const float takef = rem >= d ? 1.f : 0.f;
    const int from = ((lane + d) & 63) << 2;
#pragma unroll
    for (int nb = 0; nb < MB; ++nb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float v = acc[nb][r];
        const float t = __int_as_float(__builtin_amdgcn_ds_bpermute(from, __float_as_int(v)));
        acc[nb][r] = fmaf(t, takef, v);
      }
      // one block's exchanges at a time: all of them in flight at once would hold 16 * MB more
      // registers than the callers that keep a next tile's rows in flight can spare
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  const bool ends_tile = l32 + rem == nv - 1;
  const bool to_c0 = head && l32 == 0 && m.prev_d == m.dst;
  const bool to_c1 = head && !to_c0 && ends_tile && m.next_d == m.dst;
  const int dsel = (head && !to_c0 && !to_c1) ? m.dst : -1;      // row this lane's total goes to
  store_rows_via_lds<T, H, false>(acc, stage, lane, [&](int r) -> T * {
    const int d = __shfl(dsel, r);
    return d >= 0 ? out + (size_t)d * H : nullptr;
  });
  if (to_c0 || to_c1) {
    const int64_t crow = wt * 2 + (to_c1 ? 1 : 0);
#pragma unroll
    for (int nb = 0; nb < MB; ++nb) store_tile_rows<float, H>(carry, crow, true, nb, g, acc[nb]);
  }
}

// Node-update layer input (Section 3.4) of one node, without its one-hot block: column k of
// [sum of the node's incoming edge attributes (De) | dense attributes (Dd)], zero beyond. The
// in-edges are the node's contiguous receiver-order range [e0, e1) and are added in that order;
// the first two are requested together (most nodes of a computation graph have one or two).
struct EmbedRow {
  int op, e0, e1;
  const float *dense;
};
__device__ __forceinline__ EmbedRow load_embed_row(const int32_t *node_op, const int32_t *in_ptr,
                                                   const float *node_dense, int Dd, int64_t row) {
  EmbedRow r;
  r.op = node_op[row];
  r.e0 = in_ptr[row];
  r.e1 = in_ptr[row + 1];
  r.dense = node_dense + (size_t)row * Dd;
  return r;
}
// four consecutive columns k0 .. k0+3 (k0 a multiple of 4, as are De and the row stride)
__device__ __forceinline__ f32x4 embed_columns(const EmbedRow &r, const float *edge_feat, int De, int Dd, int k0) {
  f32x4 x = {0.f, 0.f, 0.f, 0.f};
  if (k0 < De) {
    const int n = r.e1 - r.e0;
    const float *p = edge_feat + (size_t)r.e0 * De + k0;
    f32x4 v0 = {0.f, 0.f, 0.f, 0.f}, v1 = v0;
    if (n > 0) v0 = *(const f32x4 *)p;
    if (n > 1) v1 = *(const f32x4 *)(p + De);
    x = v0;
    if (n > 1) x += v1;
    for (int e = 2; e < n; ++e) x += *(const f32x4 *)(p + (size_t)e * De);
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (k0 + j < De + Dd) x[j] = r.dense[k0 + j - De];
  }
  return x;
}

// The same four columns with every load under no condition (an absent edge, a column of the other
// kind or past the last one reads a row of zeros through the load address; up to four in-edges,
// the rest in a loop), so that no load waits for another. Sums in the order of embed_columns
// (adding the zeros changes nothing).
__device__ __forceinline__ f32x4 embed_columns_ahead(const EmbedRow &r, const float *edge_feat, const float *zeros,
                                                     int De, int Dd, int k0) {
  const int n = k0 < De ? r.e1 - r.e0 : 0;
  const float *p = edge_feat + (size_t)r.e0 * De + k0;
  f32x4 v[4], d;
#pragma unroll
  for (int e = 0; e < 4; ++e) v[e] = *(const f32x4 *)(e < n ? p + (size_t)e * De : zeros);
#pragma unroll
  for (int j = 0; j < 4; ++j) d[j] = *(k0 >= De && k0 + j < De + Dd ? r.dense + (k0 + j - De) : zeros);
  f32x4 x = v[0];
#pragma unroll
  for (int e = 1; e < 4; ++e) x += v[e];
  for (int e = 4; e < n; ++e) x += *(const f32x4 *)(p + (size_t)e * De);
  x += d;
  return x;
}

// EMBED: zero rows of the received-sum buffers for the tile's nodes without in-edges (`no_in`:
// this lane's node, lane = row l % 32), whole rows, 16 bytes per lane.
template <typename T, int H>
__device__ __forceinline__ void zero_source_rows(const Mlp2Args &a, int64_t row0, int nv, bool no_in, int lane) {
  constexpr int LPR = H * (int)sizeof(T) / 16, RPI = 64 / LPR;
  if (a.n_agg == 0 || !__any(no_in)) return;
  const int flag = no_in ? 1 : 0;
#pragma unroll
  for (int k = 0; k < 32 / RPI; ++k) {
    const int r = k * RPI + lane / LPR;
    const bool z = __shfl(flag, r) != 0 && r < nv;
    if (z)
      for (int i = 0; i < a.n_agg; ++i)
        *(f32x4 *)((char *)a.agg0 + i * a.agg_stride + ((size_t)(row0 + r) * H) * sizeof(T) + (lane % LPR) * 16) =
            f32x4{0.f, 0.f, 0.f, 0.f};
  }
}

// One wave tile: rows [row0, row0 + nv) (nv in 1..32; for EDGE the edges of tile `wt` of the
// tile table in use), staged out through `stage` (RowStage<T, H>::BYTES, private to the wave).
// T1 = operand type of layer 1 (its input rows and W1), T = operand type of layer 2 and of the
// stored activations. They differ only for EMBED in bf16 mode, whose first layer stays in fp32:
// its inputs (log2 shape attributes up to 12, sums of edge attributes) are large enough for bf16
// weight rounding to dominate the error of the whole encoder.
template <typename T1, typename T, int H, int KIND>
__device__ __forceinline__ void mlp2_wave_tile(const Mlp2Args &a, const int64_t row0, const int nv, const int64_t wt,
                                               char *stage, const int lane) {
  using Opd = Operand<T>;
  using vec = typename Opd::vec;
  constexpr int V = Opd::V, SL = 2 * V, MB = H / 32, HS = H / SL;
  using Opd1 = Operand<T1>;
  using vec1 = typename Opd1::vec;
  constexpr int V1 = Opd1::V, SL1 = 2 * V1;
  static_assert(KIND == KIND_EMBED || sizeof(T1) == sizeof(T), "only EMBED mixes operand types");
  const int l32 = lane & 31, g = lane >> 5;
  const int64_t row = row0 + (l32 < nv ? l32 : nv - 1);          // clamp loads; stores are guarded

  // ---------------- layer 1: acc1[mb] = (W1^T x^T) tile, features x rows, bias pre-loaded
  f32x16 acc1[MB];
  if constexpr (KIND != KIND_EMBED) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc1[mb][r] = a.b1[32 * mb + acc_row(r, g)];
  }
  const vec1 *W1 = (const vec1 *)(KIND == KIND_EMBED ? a.W1x : a.W1s) + lane;

  if constexpr (KIND == KIND_EDGE || KIND == KIND_NODE) {
    // both H-wide parts of the input row are requested up front (one exposed latency instead
    // of one per slab); the weight fragments are requested one slab ahead of their MFMAs
    const T *pa, *pb;
    if constexpr (KIND == KIND_EDGE) {
      pa = (const T *)a.h + (size_t)a.in_src[row] * H + g * V;
      pb = (const T *)a.h + (size_t)a.in_dst[row] * H + g * V;
    } else {
      pa = (const T *)a.h + (size_t)row * H + g * V;
      const int64_t ar = a.agg_src ? (int64_t)a.agg_src[row] : row;
      pb = ar < 0 ? (const T *)a.zero_row + g * V : (const T *)a.agg + (size_t)ar * H + g * V;
    }
    vec xa[HS], xb[HS];
#pragma unroll
    for (int s = 0; s < HS; ++s) xa[s] = *(const vec *)(pa + s * SL);
#pragma unroll
    for (int s = 0; s < HS; ++s) xb[s] = *(const vec *)(pb + s * SL);
    [[maybe_unused]] TailRaw<V> xt;
    if constexpr (KIND == KIND_EDGE) xt = load_tail<V>(a.edge_feat + (size_t)row * a.De, a.De, 0, g);
    vec wc[MB], wn[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) wc[mb] = W1[mb * 64];
#pragma unroll
    for (int s = 0; s < 2 * HS; ++s) {
      if (s + 1 < a.nslab1) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) wn[mb] = W1[((size_t)(s + 1) * MB + mb) * 64];
      }
      const vec x = s < HS ? xa[s < HS ? s : 0] : xb[s < HS ? 0 : s - HS];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) Opd::mma(wc[mb], x, acc1[mb]);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) wc[mb] = wn[mb];
    }
    if constexpr (KIND == KIND_EDGE) {
      const float *xe = a.edge_feat + (size_t)row * a.De;
      for (int s = 2 * HS; s < a.nslab1; ++s) {                 // edge attributes
        const vec x = tail_to_operand<T>(s == 2 * HS ? xt : load_tail<V>(xe, a.De, s - 2 * HS, g));
        if (s > 2 * HS) {
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) wc[mb] = W1[((size_t)s * MB + mb) * 64];
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) Opd::mma(wc[mb], x, acc1[mb]);
      }
    }
  } else {
    // The one-hot block of the input selects one row of W1: that row (plus the bias) is the
    // accumulators' starting value, read as four consecutive features per load, and only the
    // remaining [edge-attr sum | dense attrs] columns go through the matrix cores (in fp32).
    const EmbedRow er = load_embed_row(a.node_op, a.in_ptr, a.node_dense, a.Dd, row);
    const float *trow = a.table + (size_t)er.op * H + 4 * g;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f32x4 t = *(const f32x4 *)(trow + 32 * mb + 8 * q);
        const f32x4 b = *(const f32x4 *)(a.b1 + 32 * mb + 8 * q + 4 * g);
#pragma unroll
        for (int j = 0; j < 4; ++j) acc1[mb][4 * q + j] = t[j] + b[j];
      }
    static_assert(V1 == 4, "the embed MLP's first layer uses fp32 operands");
    for (int s = 0; s < a.nslabx; ++s) {
      const vec1 x = embed_columns(er, a.edge_feat, a.De, a.Dd, s * SL1 + g * V1);
      mma_slab<T1, H>(W1 + (size_t)s * MB * 64, x, acc1);
    }
  }

  // ---------------- layer 2, transposed as well: acc2[nb] = (W2^T relu(z1)^T) tile, features x
  // rows, bias pre-loaded. Lane = row, and a lane's register quads are four consecutive features
  // of its row: 8- or 16-byte stores, and for EDGE a per-receiver sum across adjacent lanes.
  f32x16 acc2[MB];
#pragma unroll
  for (int nb = 0; nb < MB; ++nb) {
#pragma unroll
    for (int r = 0; r < 16; ++r) acc2[nb][r] = a.b2[32 * nb + acc_row(r, g)];
  }
  const vec *W2 = (const vec *)a.W2s + lane;
  {
    constexpr int QB = 32 / SL, NC2 = MB * QB;
    vec wc[MB], wn[MB];
#pragma unroll
    for (int nb = 0; nb < MB; ++nb) wc[nb] = W2[nb * 64];
#pragma unroll
    for (int c = 0; c < NC2; ++c) {
      if (c + 1 < NC2) {
#pragma unroll
        for (int nb = 0; nb < MB; ++nb) wn[nb] = W2[((size_t)(c + 1) * MB + nb) * 64];
      }
      const vec z = relu_operand<T>(acc1[c / QB], c % QB);
#pragma unroll
      for (int nb = 0; nb < MB; ++nb) Opd::mma(wc[nb], z, acc2[nb]);
#pragma unroll
      for (int nb = 0; nb < MB; ++nb) wc[nb] = wn[nb];
    }
  }

  // ---------------- epilogue
  T *out = (T *)a.out;
  if constexpr (KIND != KIND_EDGE) {
    store_rows_via_lds<T, H, true>(acc2, stage, lane, [&](int r) -> T * {
      return r < nv ? out + (size_t)(row0 + r) * H : nullptr;
    });
    if constexpr (KIND == KIND_EMBED) zero_source_rows<T, H>(a, row0, nv, a.in_ptr[row + 1] == a.in_ptr[row], lane);
  } else {
    const EdgeTileMeta m = load_edge_meta(a.in_dst, a.n_rows, row0, nv, l32);
    edge_tile_sum<T, H>(acc2, m, wt, nv, lane, out, a.carry, stage);
  }
}

// Streaming form: one block of four waves per 128 rows (four edge tiles), weights read from
// memory (L2) as they are needed.
template <typename T1, typename T, int H, int KIND>
__global__ __launch_bounds__(256) void mlp2_kernel(const Mlp2Args a) {
  __shared__ __align__(16) char stage[4][RowStage<T, H>::BYTES];  // per-wave staging of output rows
  // consecutive tiles stay on one XCD (blocks are dealt round-robin to the 8 XCDs), so the rows
  // a tile gathers are mostly in that XCD's L2 already
  const int64_t per_xcd = (a.n_blocks + 7) / 8;
  const int64_t tile = (int64_t)(blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (tile >= a.n_blocks) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t wt = tile * 4 + wave;                           // wave tile: 32 rows, or an edge tile
  int64_t row0 = wt * 32;
  int nv;
  if constexpr (KIND == KIND_EDGE) {
    if (wt >= a.n_tiles) return;
    row0 = a.tile_ptr[wt];
    nv = a.tile_ptr[wt + 1] - (int)row0;
  } else {
    if (row0 >= a.n_rows) return;
    nv = a.n_rows - row0 < 32 ? (int)(a.n_rows - row0) : 32;
  }
  mlp2_wave_tile<T1, T, H, KIND>(a, row0, nv, wt, stage[wave], lane);
}
