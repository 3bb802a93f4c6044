// Persistent variant of the fused two-layer MLP (edge and node kinds) for operand widths whose
// fragment-ordered weights fit in LDS (bf16, H <= 128: at most 104 KB of the CU's 160 KB):
// one block of NW waves per CU copies both weight matrices into LDS once and then walks over
// wave tiles of 32 rows, so the steady state reads weights from LDS only and rows from memory.
// Wave tiles are dealt to waves one at a time (not in block-sized groups), so a problem of only a
// few tiles per CU still spreads evenly.
//
// Each wave loads the rows of its tile, computes and stores; the two waves that share a SIMD
// overlap one's loads and epilogue with the other's MFMAs. A wave's requests run ahead of its
// arithmetic: the edge range of the tile after next, the row indices of the next tile, and, once
// layer 2 has freed the registers, the next tile's rows. (More than 8 waves per CU do not fit the
// register file at H = 128 without spilling and measured slower.)
// Inside a layer the weight fragments of the next contraction slab are read from LDS while the
// MFMAs of the current slab run. Math, operand layouts and epilogues are those of mlp2_kernel.
#pragma once
#include "mlp2.hip.h"

template <typename T, int H>
struct TileRows {
  using vec = typename Operand<T>::vec;
  static constexpr int NX = 2 * (H / (2 * Operand<T>::V));   // slabs of the two H-wide parts
  vec x[NX];
  TailRaw<Operand<T>::V> xe;   // EDGE: the single slab of edge attributes as requested (not yet zero-padded)
};

struct TileIndex {
  int e0, nv;       // EDGE: the tile's edges are [e0, e0 + nv)
  int src;          // EDGE: sender of this lane's edge; NODE: row of the received sums to read, -1 = none
  EdgeTileMeta m;   // EDGE: receivers
};

struct TileBounds {
  int e0, e1;       // EDGE: the tile's edges are [e0, e1); NODE: e0 = first node of the tile
};
template <int KIND>
__device__ __forceinline__ TileBounds load_bounds(const Mlp2Args &a, int64_t wt) {
  TileBounds b{0, 0};
  if constexpr (KIND == KIND_EDGE) {
    b.e0 = a.tile_ptr[wt];
    b.e1 = a.tile_ptr[wt + 1];
  } else {
    b.e0 = (int)(wt * 32);
  }
  return b;
}
template <int KIND>
__device__ __forceinline__ TileIndex load_index(const Mlp2Args &a, const TileBounds &b, int l32) {
  TileIndex ix;
  if constexpr (KIND == KIND_EDGE) {
    ix.e0 = b.e0;
    ix.nv = b.e1 - b.e0;
    ix.src = a.in_src[ix.e0 + (l32 < ix.nv ? l32 : ix.nv - 1)];
    ix.m = load_edge_meta(a.in_dst, a.n_rows, ix.e0, ix.nv, l32);
  } else {
    const int64_t row = (int64_t)b.e0 + l32 < a.n_rows ? (int64_t)b.e0 + l32 : a.n_rows - 1;
    ix.e0 = b.e0;
    ix.nv = 0;
    ix.src = a.agg_src[row];   // (must be given: a load under a condition would be waited for on the spot)
  }
  return ix;
}

// Issues the row loads of a wave tile: PARTS & 1 the first H-wide part (EDGE: the sender's row,
// NODE: the node's own), PARTS & 2 the second (EDGE: the receiver's row and the edge attributes,
// NODE: the received sum). All loads are unconditional (clamped) so none waits on another.
template <typename T, int H, int KIND, int PARTS>
__device__ __forceinline__ void load_rows(const Mlp2Args &a, int64_t wt, int l32, int g, const TileIndex &ix,
                                          TileRows<T, H> &in) {
  using Opd = Operand<T>;
  using vec = typename Opd::vec;
  constexpr int V = Opd::V, SL = 2 * V, HS = H / SL;
  if constexpr (KIND == KIND_EDGE) {
    if constexpr ((PARTS & 1) != 0) {
      const T *hs = (const T *)a.h + (size_t)ix.src * H + g * V;
#pragma unroll
      for (int k = 0; k < HS; ++k) in.x[k] = *(const vec *)(hs + k * SL);
    }
    if constexpr ((PARTS & 2) != 0) {
      const int64_t row = ix.e0 + (l32 < ix.nv ? l32 : ix.nv - 1);
      const T *hd = (const T *)a.h + (size_t)ix.m.dst * H + g * V;
#pragma unroll
      for (int k = 0; k < HS; ++k) in.x[HS + k] = *(const vec *)(hd + k * SL);
      in.xe = request_tail<V>(a.edge_feat + (size_t)row * a.De, a.De, 0, g);
    }
  } else {
    int64_t row = wt * 32 + l32;
    if (row >= a.n_rows) row = a.n_rows - 1;
    if constexpr ((PARTS & 1) != 0) {
      const T *hp = (const T *)a.h + (size_t)row * H + g * V;
#pragma unroll
      for (int k = 0; k < HS; ++k) in.x[k] = *(const vec *)(hp + k * SL);
    }
    if constexpr ((PARTS & 2) != 0) {
      const T *ap = ix.src < 0 ? (const T *)a.zero_row + g * V : (const T *)a.agg + (size_t)ix.src * H + g * V;
#pragma unroll
      for (int k = 0; k < HS; ++k) in.x[HS + k] = *(const vec *)(ap + k * SL);
    }
  }
}

// Layer 2 of a wave tile with the weights in LDS: acc2 = W2^T relu(z1)^T + b2 (features x rows);
// the fragments of the next chunk are read while the MFMAs of the current one run.
template <typename T, int H>
__device__ __forceinline__ void layer2_lds(const f32x16 (&acc1)[H / 32], const typename Operand<T>::vec *W2l,
                                           const float (*b2l)[2][16], int lane, int g, f32x16 (&acc2)[H / 32]) {
  using Opd = Operand<T>;
  using vec = typename Opd::vec;
  constexpr int MB = H / 32, QB = 32 / (2 * Opd::V), NC2 = MB * QB;
#pragma unroll
  for (int nb = 0; nb < MB; ++nb) acc2[nb] = *(const f32x16 *)&b2l[nb][g][0];
  vec wc[MB];
#pragma unroll
  for (int nb = 0; nb < MB; ++nb) wc[nb] = W2l[nb * 64 + lane];
#pragma unroll
  for (int c = 0; c < NC2; ++c) {
    vec wn[MB];
    if (c + 1 < NC2) {
#pragma unroll
      for (int nb = 0; nb < MB; ++nb) wn[nb] = W2l[((c + 1) * MB + nb) * 64 + lane];
    }
    const vec z = relu_operand<T>(acc1[c / QB], c % QB);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int nb = 0; nb < MB; ++nb) Opd::mma(wc[nb], z, acc2[nb]);
    __builtin_amdgcn_sched_barrier(0);
    if (c + 1 < NC2) {
#pragma unroll
      for (int nb = 0; nb < MB; ++nb) wc[nb] = wn[nb];
    }
  }
}

// The same product for half of the output feature blocks (nb0 .. nb0 + H / 64 - 1) from relu(z1)
// already converted to operand fragments: with H = 256 the two full sets of fp32 accumulators and
// the weight fragments in flight do not fit a wave's 256 registers, fragments (a quarter of the
// accumulators' size) plus half of the outputs do. Every output accumulates its chunks in the
// order of layer2_lds, so the results are the same bits.
template <typename T, int H>
__device__ __forceinline__ void layer2_half_lds(const typename Operand<T>::vec (&zf)[H / (2 * Operand<T>::V)],
                                                const typename Operand<T>::vec *W2l, const float (*b2l)[2][16], int lane,
                                                int g, int nb0, f32x16 (&acc2)[H / 64]) {
  using Opd = Operand<T>;
  using vec = typename Opd::vec;
  constexpr int MB = H / 32, HB = MB / 2, NC2 = H / (2 * Opd::V);
#pragma unroll
  for (int i = 0; i < HB; ++i) acc2[i] = *(const f32x16 *)&b2l[nb0 + i][g][0];
  vec wc[HB];
#pragma unroll
  for (int i = 0; i < HB; ++i) wc[i] = W2l[(nb0 + i) * 64 + lane];
#pragma unroll
  for (int c = 0; c < NC2; ++c) {
    vec wn[HB];
    if (c + 1 < NC2) {
#pragma unroll
      for (int i = 0; i < HB; ++i) wn[i] = W2l[((c + 1) * MB + nb0 + i) * 64 + lane];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < HB; ++i) Opd::mma(wc[i], zf[c], acc2[i]);
    __builtin_amdgcn_sched_barrier(0);
    if (c + 1 < NC2) {
#pragma unroll
      for (int i = 0; i < HB; ++i) wc[i] = wn[i];
    }
  }
}

// What a SAVE kernel keeps for the backward pass from a wave tile held as features x rows
// accumulators (lane = row). Before layer 2 (which consumes layer 1's accumulators block by block,
// so they need not stay live beyond it): relu(z1) rows [row0, row0 + nv) of a.z1 through the
// staging buffer, one 32-feature block at a time with BLOCKWISE staging, else whole rows.
template <typename T, int H, bool BLOCKWISE>
__device__ __forceinline__ void save_hidden_tile(const Mlp2Args &a, const f32x16 (&acc1)[H / 32], int64_t wt, int64_t row0,
                                                 int nv, int lane, char *stage) {
  constexpr int MB = H / 32;
  T *z1 = (T *)a.z1;
  {
    int lv = lane;                      // (opaque: the address is formed here, not kept in registers across tiles)
    asm volatile("" : "+v"(lv));
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) a.z1mask[((size_t)wt * MB + mb) * 64 + lv] = lane_mask_bits(acc1[mb]);
  }
  if constexpr (BLOCKWISE) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      f32x16 d;
#pragma unroll
      for (int r = 0; r < 16; ++r) d[r] = relu_f32(acc1[mb][r]);
      store_block_via_lds<T, H>(z1, row0, nv, mb, lane, d, stage);
    }
  } else {
    store_rows_via_lds<T, H, true>(acc1, stage, lane, [&](int r) -> T * {
      return r < nv ? z1 + (size_t)(row0 + r) * H : nullptr;
    });
  }
}
// After layer 2 (tile wt): the mask bits of y.
template <int H>
__device__ __forceinline__ void save_output_mask(const Mlp2Args &a, const f32x16 (&acc2)[H / 32], int64_t wt, int lane) {
  int lv = lane;                        // (opaque: the address is formed here, not kept in registers across tiles)
  asm volatile("" : "+v"(lv));
#pragma unroll
  for (int nb = 0; nb < H / 32; ++nb) a.ymask[((size_t)wt * (H / 32) + nb) * 64 + lv] = lane_mask_bits(acc2[nb]);
}

template <typename T, int H, int KIND, int NW, bool SAVE>
__global__ __launch_bounds__(64 * NW) void mlp2p_kernel(const Mlp2Args a) {
  using Opd = Operand<T>;
  using vec = typename Opd::vec;
  constexpr int V = Opd::V, SL = 2 * V, MB = H / 32, HS = H / SL, QB = 32 / SL;
  constexpr int NS1 = 2 * HS + (KIND == KIND_EDGE ? 1 : 0);   // slabs of layer 1
  constexpr int NC2 = MB * QB;                                // chunks of layer 2
  static_assert(KIND == KIND_EDGE || KIND == KIND_NODE, "the embed MLP has its own kernel below");
  extern __shared__ __align__(16) char smem[];
  vec *W1l = (vec *)smem;                                  // [NS1][MB][64]
  vec *W2l = W1l + (size_t)NS1 * MB * 64;                  // [NC2][MB][64]
  float(*b1l)[2][16] = (float(*)[2][16])(W2l + (size_t)NC2 * MB * 64);   // [MB][lane group][16]
  float(*b2l)[2][16] = b1l + MB;                                         // same for layer 2
  char *stage = (char *)(b2l + MB) + (threadIdx.x >> 6) * RowStage<T, H>::BYTES;   // this wave's output staging

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // tile counters stay in scalar registers
  // the wave tiles of one XCD are contiguous (blocks are dealt round-robin to the 8 XCDs); inside
  // the XCD, tile j of a pass goes to wave j / nbx of block j % nbx
  const int nbx = gridDim.x / 8, xcd = blockIdx.x % 8, lid = blockIdx.x / 8;
  const int64_t n_wt = KIND == KIND_EDGE ? a.n_tiles : (a.n_rows + 31) / 32;
  const int64_t per_xcd = (n_wt + 7) / 8;
  const int64_t t_begin = xcd * per_xcd;
  const int64_t t_end = (t_begin + per_xcd) < n_wt ? (t_begin + per_xcd) : n_wt;
  const int64_t stride = (int64_t)nbx * NW;
  int64_t wt = t_begin + (int64_t)wave * nbx + lid;

  // Start-up: request the first tile's indices, then all of this thread's share of the weights
  // in one batch of loads (a load-store loop would pay one memory round trip per 8 KB), and only
  // then move the weights into LDS.
  TileIndex ix;
  TileBounds bnext;   // of the wave's next tile (of its last one again when there is no next)
  if (wt < t_end) {
    ix = load_index<KIND>(a, load_bounds<KIND>(a, wt), l32);
    bnext = load_bounds<KIND>(a, wt + stride < t_end ? wt + stride : wt);
  }
  {
    constexpr int NT = 64 * NW, N1 = NS1 * MB * 64, N2 = NC2 * MB * 64;
    constexpr int C1 = (N1 + NT - 1) / NT, C2 = (N2 + NT - 1) / NT;
    const vec *s1 = (const vec *)a.W1s, *s2 = (const vec *)a.W2s;
    vec t1[C1], t2[C2];
#pragma unroll
    for (int c = 0; c < C1; ++c) t1[c] = s1[tid + c * NT < N1 ? tid + c * NT : 0];
#pragma unroll
    for (int c = 0; c < C2; ++c) t2[c] = s2[tid + c * NT < N2 ? tid + c * NT : 0];
    float bb1 = 0.f, bb2 = 0.f;
    if (tid < MB * 32) {                                     // biases in accumulator order
      bb1 = a.b1[32 * (tid / 32) + acc_row(tid % 16, (tid / 16) % 2)];
      bb2 = a.b2[32 * (tid / 32) + acc_row(tid % 16, (tid / 16) % 2)];
    }
#pragma unroll
    for (int c = 0; c < C1; ++c)
      if (tid + c * NT < N1) W1l[tid + c * NT] = t1[c];
#pragma unroll
    for (int c = 0; c < C2; ++c)
      if (tid + c * NT < N2) W2l[tid + c * NT] = t2[c];
    if (tid < MB * 32) {
      b1l[tid / 32][(tid / 16) % 2][tid % 16] = bb1;
      b2l[tid / 32][(tid / 16) % 2][tid % 16] = bb2;
    }
  }
  __syncthreads();

  // The rows of a wave's next tile are requested once layer 2 has consumed layer 1's accumulators
  // (the registers of the current rows and of those accumulators are free from there on), so the
  // gather's round trip runs under the epilogue; the next tile's indices are requested a tile
  // earlier and its edge range a tile before that, so no request waits on another's answer.
  TileRows<T, H> in;
  if (wt < t_end) load_rows<T, H, KIND, 3>(a, wt, l32, g, ix, in);
  for (; wt < t_end; wt += stride) {
    // the weights in LDS never change, but keeping all their fragments in registers across
    // tiles would not fit: make the compiler re-read them from LDS in every tile
    asm volatile("" ::: "memory");
    [[maybe_unused]] const EdgeTileMeta meta = ix.m;
    [[maybe_unused]] const int nv = ix.nv;
    [[maybe_unused]] const int64_t meta_e0 = ix.e0;
    const bool more = wt + stride < t_end;
    const int64_t wnext = more ? wt + stride : wt;
    ix = load_index<KIND>(a, bnext, l32);
    bnext = load_bounds<KIND>(a, wnext + stride < t_end ? wnext + stride : wnext);
    // ---------------- layer 1 (features x rows)
    f32x16 acc1[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) acc1[mb] = *(const f32x16 *)&b1l[mb][g][0];
    [[maybe_unused]] vec xe;
    if constexpr (KIND == KIND_EDGE) xe = tail_to_operand<T>(zero_tail_beyond<V>(in.xe, a.De, 0, g));
    {
      vec wc[MB];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) wc[mb] = W1l[mb * 64 + lane];
#pragma unroll
      for (int s = 0; s < NS1; ++s) {
        vec wn[MB];
        if (s + 1 < NS1) {
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) wn[mb] = W1l[((s + 1) * MB + mb) * 64 + lane];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          if (KIND == KIND_EDGE && s == 2 * HS) Opd::mma(wc[mb], xe, acc1[mb]);
          else Opd::mma(wc[mb], in.x[s < 2 * HS ? s : 0], acc1[mb]);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (s + 1 < NS1) {
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) wc[mb] = wn[mb];
        }
      }
    }
    // ---------------- layer 2 (features x rows)
    f32x16 acc2[MB];
    if constexpr (SAVE) {
      if constexpr (KIND == KIND_NODE) {
        const int64_t left = a.n_rows - wt * 32;
        save_hidden_tile<T, H, false>(a, acc1, wt, wt * 32, left < 32 ? (int)left : 32, lane, stage);
      } else {
        save_hidden_tile<T, H, false>(a, acc1, wt, meta_e0, nv, lane, stage);
      }
    }
    layer2_lds<T, H>(acc1, W2l, b2l, lane, g, acc2);
    if constexpr (SAVE) save_output_mask<H>(a, acc2, wt, lane);
    if (more) load_rows<T, H, KIND, 3>(a, wnext, l32, g, ix, in);
    else in = TileRows<T, H>{};   // (so that the consumed rows need not stay live up to here)
    __builtin_amdgcn_sched_barrier(0);
    // ---------------- epilogue
    T *out = (T *)a.out;
    if constexpr (KIND == KIND_NODE) {
      const int64_t row0 = wt * 32;
      store_rows_via_lds<T, H, true>(acc2, stage, lane, [&](int r) -> T * {
        return row0 + r < a.n_rows ? out + (size_t)(row0 + r) * H : nullptr;
      });
    } else {
      edge_tile_sum<T, H>(acc2, meta, wt, nv, lane, out, a.carry, stage);
    }
  }
}

// The node-update layer's MLP (Section 3.4) in the same persistent form. Its first layer needs
// little LDS -- the fp32 fragments for the [edge-attr sum | dense attrs] columns and the [Tn, H]
// table of W1's one-hot rows -- so two blocks fit a CU. At most 4 * 64 * NW 16-byte pieces each
// for the first-layer fragments and for the table (the launcher checks).
// At H = 256 the second layer's weights alone take 128 KB: the table then stays in global memory
// (32 KB, read through the caches), the block has four waves, and the rows leave through a
// staging buffer of one 32-feature block per wave.
template <typename T, int H, int NW, bool SAVE>
__global__ __launch_bounds__(64 * NW) void embedp_kernel(const Mlp2Args a) {
  using Opd = Operand<T>;
  using vec = typename Opd::vec;
  constexpr int V = Opd::V, SL = 2 * V, MB = H / 32, QB = 32 / SL, NC2 = MB * QB, NT = 64 * NW;
  extern __shared__ __align__(16) char smem[];
  vec *W2l = (vec *)smem;                                              // [NC2][MB][64]
  f32x4 *W1l = (f32x4 *)(W2l + (size_t)NC2 * MB * 64);                 // [nslabx][MB][64]
  constexpr bool BIG = H > 128;                                        // table in global memory, block staging
  f32x4 *tabl = W1l + (size_t)a.nslabx * MB * 64;                      // [Tn][H / 4] (not BIG)
  const f32x4 *tab = BIG ? (const f32x4 *)a.table : tabl;
  float(*b1l)[2][16] = (float(*)[2][16])(tabl + (BIG ? 0 : (size_t)a.Tn * (H / 4)));
  float(*b2l)[2][16] = b1l + MB;
  char *stage = (char *)(b2l + MB) + (threadIdx.x >> 6) * (BIG ? BlockStage<T>::BYTES : RowStage<T, H>::BYTES);

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // tile counters stay in scalar registers
  const int nbx = gridDim.x / 8, xcd = blockIdx.x % 8, lid = blockIdx.x / 8;
  const int64_t n_wt = (a.n_rows + 31) / 32;
  const int64_t per_xcd = (n_wt + 7) / 8;
  const int64_t t_begin = xcd * per_xcd;
  const int64_t t_end = (t_begin + per_xcd) < n_wt ? (t_begin + per_xcd) : n_wt;
  const int64_t stride = (int64_t)nbx * NW;
  int64_t wt = t_begin + (int64_t)wave * nbx + lid;
  {
    constexpr int N2 = NC2 * MB * 64, C2 = (N2 + NT - 1) / NT;
    const int n1 = a.nslabx * MB * 64, nt = BIG ? 0 : a.Tn * (H / 4);
    const vec *s2 = (const vec *)a.W2s;
    const f32x4 *s1 = (const f32x4 *)a.W1x, *st = (const f32x4 *)a.table;
    vec t2[C2];
    f32x4 t1[4], tt[4];
#pragma unroll
    for (int c = 0; c < C2; ++c) t2[c] = s2[tid + c * NT < N2 ? tid + c * NT : 0];
#pragma unroll
    for (int c = 0; c < 4; ++c) t1[c] = s1[tid + c * NT < n1 ? tid + c * NT : 0];
#pragma unroll
    for (int c = 0; c < 4; ++c) tt[c] = st[tid + c * NT < nt ? tid + c * NT : 0];
    float bb1 = 0.f, bb2 = 0.f;
    if (tid < MB * 32) {
      bb1 = a.b1[32 * (tid / 32) + acc_row(tid % 16, (tid / 16) % 2)];
      bb2 = a.b2[32 * (tid / 32) + acc_row(tid % 16, (tid / 16) % 2)];
    }
#pragma unroll
    for (int c = 0; c < C2; ++c)
      if (tid + c * NT < N2) W2l[tid + c * NT] = t2[c];
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (tid + c * NT < n1) W1l[tid + c * NT] = t1[c];
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (tid + c * NT < nt) tabl[tid + c * NT] = tt[c];
    if (tid < MB * 32) {
      b1l[tid / 32][(tid / 16) % 2][tid % 16] = bb1;
      b2l[tid / 32][(tid / 16) % 2][tid % 16] = bb2;
    }
  }
  __syncthreads();

  // Everything a tile reads from memory is requested a tile ahead (its row data -- op type, in-edge
  // range -- two tiles ahead) and has arrived before the previous tile's first store: loads and
  // stores complete in order, so a load requested behind a tile's stores would not be there before
  // they are, and a wave that is alone on its SIMD (H = 256) would sit through every drain.
  auto tile_row = [&](int64_t t) {
    const int64_t r = t * 32 + l32;
    return r < a.n_rows ? r : a.n_rows - 1;
  };
  auto next_tile = [&](int64_t t) { return t + stride < t_end ? t + stride : t; };
  constexpr int NSX = 2;                             // slabs of fp32 input columns at most (the launcher checks)
  f32x4 xs[NSX];                                     // the tile's fp32 input columns, one vector per slab
  [[maybe_unused]] f32x16 pre[BIG ? MB : 1];         // BIG: the op type's table row
  auto request = [&](const EmbedRow &r) {
    int gv = g;                         // (opaque: the columns' offsets are formed here in every tile instead of
    asm volatile("" : "+v"(gv));        //  living in registers, of which the loop has none to spare)
#pragma unroll
    for (int sl = 0; sl < NSX; ++sl)
      if (sl < a.nslabx) xs[sl] = embed_columns_ahead(r, a.edge_feat, (const float *)a.zero_row, a.De, a.Dd, sl * 8 + gv * 4);
    if constexpr (BIG) {
      const f32x4 *trow = tab + (size_t)r.op * (H / 4) + gv;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x4 t = trow[8 * mb + 2 * q];
#pragma unroll
          for (int j = 0; j < 4; ++j) pre[mb][4 * q + j] = t[j];
        }
    }
  };
  EmbedRow er = load_embed_row(a.node_op, a.in_ptr, a.node_dense, a.Dd, tile_row(wt < t_end ? wt : 0));
  EmbedRow er_next = load_embed_row(a.node_op, a.in_ptr, a.node_dense, a.Dd, tile_row(wt < t_end ? next_tile(wt) : 0));
  request(er);
  auto arrived = [&]() {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0x0F70);                        // vmcnt(0)
    __builtin_amdgcn_sched_barrier(0);
  };
  arrived();
  for (; wt < t_end; wt += stride) {
    asm volatile("" ::: "memory");
    const int64_t row0 = wt * 32;
    const int64_t left = a.n_rows - row0;
    const int n_valid = left < 32 ? (int)left : 32;
    // ---------------- layer 1: bias + the op type's row of W1, then the fp32 columns on the MFMAs
    f32x16 acc1[MB];
    if constexpr (BIG) {
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const f32x16 b = *(const f32x16 *)&b1l[mb][g][0];
#pragma unroll
        for (int r = 0; r < 16; ++r) acc1[mb][r] = pre[mb][r] + b[r];
      }
    } else {
      const f32x4 *trow = tab + (size_t)er.op * (H / 4) + g;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        acc1[mb] = *(const f32x16 *)&b1l[mb][g][0];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x4 t = trow[8 * mb + 2 * q];
#pragma unroll
          for (int j = 0; j < 4; ++j) acc1[mb][4 * q + j] += t[j];
        }
      }
    }
#pragma unroll
    for (int sl = 0; sl < NSX; ++sl)
      if (sl < a.nslabx) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) Operand<float>::mma(W1l[(sl * MB + mb) * 64 + lane], xs[sl], acc1[mb]);
      }
    // ---------------- the next tile's requests (its row data arrived a tile ago)
    er = er_next;
    request(er);
    er_next = load_embed_row(a.node_op, a.in_ptr, a.node_dense, a.Dd, tile_row(next_tile(next_tile(wt))));
    T *out = (T *)a.out;
    if constexpr (BIG) {
      // relu(z1) as operand fragments first (they are also what is kept of it), then the output
      // feature blocks in two halves, each leaving through the staging buffer before the other
      // is formed. The first half's products run under the requests' round trip; nothing is
      // stored before they have arrived.
      constexpr int HB = MB / 2;
      [[maybe_unused]] uint16_t zbits[MB];
      if constexpr (SAVE) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) zbits[mb] = lane_mask_bits(acc1[mb]);
      }
      vec zf[NC2];
#pragma unroll
      for (int c = 0; c < NC2; ++c) zf[c] = relu_operand<T>(acc1[c / QB], c % QB);
#pragma unroll
      for (int hb = 0; hb < 2; ++hb) {
        f32x16 acc2[HB];
        layer2_half_lds<T, H>(zf, W2l, b2l, lane, g, hb * HB, acc2);
        if (hb == 0) {
          arrived();
          if constexpr (SAVE) {
            int lv = lane;              // (opaque: the address is formed here, not kept in registers across tiles)
            asm volatile("" : "+v"(lv));
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) a.z1mask[((size_t)wt * MB + mb) * 64 + lv] = zbits[mb];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
              store_block_fragments_via_lds<H>((T *)a.z1, row0, n_valid, mb, lv, zf[2 * mb], zf[2 * mb + 1], stage);
          }
        }
        int lv = lane;                  // (opaque, as above)
        asm volatile("" : "+v"(lv));
        if constexpr (SAVE) {
#pragma unroll
          for (int i = 0; i < HB; ++i) a.ymask[((size_t)wt * MB + hb * HB + i) * 64 + lv] = lane_mask_bits(acc2[i]);
        }
#pragma unroll
        for (int i = 0; i < HB; ++i) {
#pragma unroll
          for (int r = 0; r < 16; ++r) acc2[i][r] = relu_f32(acc2[i][r]);
          store_block_via_lds<T, H>(out, row0, n_valid, hb * HB + i, lv, acc2[i], stage);
        }
      }
    } else {
      arrived();                                             // before the first store (as above)
      if constexpr (SAVE) save_hidden_tile<T, H, false>(a, acc1, wt, row0, n_valid, lane, stage);
      f32x16 acc2[MB];
      layer2_lds<T, H>(acc1, W2l, b2l, lane, g, acc2);
      if constexpr (SAVE) save_output_mask<H>(a, acc2, wt, lane);
      store_rows_via_lds<T, H, true>(acc2, stage, lane, [&](int r) -> T * {
        return row0 + r < a.n_rows ? out + (size_t)(row0 + r) * H : nullptr;
      });
    }
  }
}
