// Backward of the fused two-layer ReLU MLPs from what the forward pass kept (Section 3.3.4: one
// back-propagation through the GNN of Section 3.4), bf16, for the batches whose forward kernels
// store the ReLU masks of the hidden pre-activation z1 and of the output y as bits (16 per lane,
// 32-feature block and wave tile) next to the hidden activation relu(z1) [rows, H] that the weight
// gradient needs. With the bits the backward needs no forward arithmetic, no gathered input rows
// and no activation rows at all:
//     dz2 = dy * [y > 0],  dz1 = (dz2 W2^T) * [z1 > 0],  dx = dz1 W1^T
// dz2 and dz1 are stored for the weight-gradient kernel, which reads relu(z1) from the forward's
// copy. Everything is kept transposed
// (features x rows: lane = row, registers = features), each result already laid out as the next
// contraction's B operand, as in mlp2_bwd_kernel; the three live tiles of that kernel (z1, dz2,
// dz1) shrink to two, which lets eight waves share a compute unit at H = 256. The weights go
// through the same double-buffered LDS groups, fetched once per block of NW waves. A wave's tile
// is the forward kernel's wave tile, because the mask bits are per tile and lane of that kernel: 32
// consecutive nodes, or for EDGE an edge tile of the packer (at most 32 edges). Those tiles are cut at receiver
// boundaries, so with FOLD (batches in which no receiver has more than 32 in-edges) the gradients
// w.r.t. h_receiver are summed per receiver across the lanes of the tile, as the forward sums the
// messages, and leave as one row per receiver instead of one per edge.
#pragma once
#include "mlp2_bwd.hip.h"

struct Mlp2BwdzArgs {
  int64_t n_rows, n_blocks;
  const void *W2bt, *W1bt;     // contraction over the weight's columns (see swizzle_chain)
  const void *dy;              // upstream gradient [N, H] bf16 (EDGE: indexed by receiver); kernels instantiated
                               // with GIVEN: dz2 itself, already masked by [y > 0] (then ymask and dz2 are unused)
  const int32_t *dy_index;     // NODE, EMBED, optional: row n reads dy[dy_index[n]] (the gradient of the
                               // per-graph sum, one row per graph, for the layer the readout sums)
  const uint16_t *z1mask;      // [tiles][H / 32][64] mask bits of z1 and of y, kept by the forward (see
  const uint16_t *ymask;       //   Mlp2Args); tiles = the edge tiles (EDGE), else 32 consecutive rows
  const int32_t *agg_src;      // [N] (NODE) negative for a node without in-edges: its row of dx_b, the gradient
                               // w.r.t. a received sum that nobody sent, is not stored (nobody reads it)
  const int32_t *in_dst;       // [E] (EDGE)
  const int32_t *tile_ptr;     // [n_tiles + 1] (EDGE)
  int64_t n_tiles;             // (EDGE)
  void *dz1, *dz2;             // [rows, H] bf16
  void *dx_a, *dx_b;           // EDGE: d h_sender, d h_receiver [E, H]; NODE: d h, d agg [N, H]; EMBED: unused
                               // EDGE with FOLD: dx_b [N, H] = d h_receiver summed per receiver (rows of
                               // receivers without in-edges are not written)
};

// Weight fragments for NW waves, UG units of UF fragments per group, through LDS: every wave
// fetches GF / NW of a group's fragments a whole group ahead of their use.
template <int UF, int UG, int NW>
struct WeightGroupsN {
  static constexpr int GF = UF * UG, PW = GF / NW;
  static_assert(GF % NW == 0, "a group is fetched by all waves of the block");
  f32x4 (*buf)[GF][64];
  int p = 0, wave, lane;
  f32x4 r[PW];
  template <typename Idx>
  __device__ __forceinline__ void fetch(const bf16x8 *W, Idx idx) {
#pragma unroll
    for (int i = 0; i < PW; ++i) {
      const int jg = wave * PW + i;
      r[i] = __builtin_bit_cast(f32x4, W[(size_t)idx(jg / UF, jg % UF) * 64]);
    }
  }
  __device__ __forceinline__ void commit(int q) {
#pragma unroll
    for (int i = 0; i < PW; ++i) buf[q][wave * PW + i][lane] = r[i];
  }
  template <typename Idx>
  __device__ __forceinline__ void begin(const bf16x8 *W, Idx idx) {
    fetch(W, idx);
    commit(p);
    __syncthreads();
  }
  __device__ __forceinline__ void next(bool have_next) {
    if (have_next) commit(p ^ 1);
    __syncthreads();
    p ^= 1;
  }
  __device__ __forceinline__ bf16x8 get(int u, int j) const { return __builtin_bit_cast(bf16x8, buf[p][u * UF + j][lane]); }
};

template <int H>
struct BwdzShape {
  static constexpr int NW = H >= 256 ? 8 : 4;                 // waves per block
  static constexpr int MB = H / 32, QB = 2, UF = MB * QB;     // 32-feature blocks, slabs per block, fragments per unit
  static constexpr int UG = H >= 256 ? 4 : 2;                 // units per group
  static constexpr size_t LDS = (size_t)NW * BlockStage<bf16_t>::BYTES + 2 * (size_t)(UF * UG) * 1024;
};

// One block per group of NW tiles, one tile per wave. (A persistent form -- as many blocks as are
// resident at once, each looping over its share with the next group's mask bits and dy rows
// requested a product ahead -- measured slower: 11.5 against 9.9 ms for the node MLP of the largest
// configuration.)
// GIVEN (NODE, EMBED): the kernel that produced the upstream gradient has already applied [y > 0]
// and left the result where the weight gradient reads dz2, so it is neither masked nor stored here.
template <int H, int KIND, bool FOLD, bool GIVEN = false>
__global__ __launch_bounds__((64 * BwdzShape<H>::NW)) void mlp2_bwdz_kernel(const Mlp2BwdzArgs a) {
  static_assert(!FOLD || KIND == KIND_EDGE, "only the edge MLP's receiver-side gradients are summed");
  static_assert(!GIVEN || KIND != KIND_EDGE, "the edge MLP's upstream gradient is gathered per receiver");
  using T = bf16_t;
  using S = BwdzShape<H>;
  using BS = BlockStage<T>;
  constexpr int MB = S::MB, QB = S::QB, UF = S::UF, UG = S::UG, NW = S::NW;
  using WG = WeightGroupsN<UF, UG, NW>;
  const int64_t per_xcd = (a.n_blocks + 7) / 8;
  const int64_t tile = (int64_t)(blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (tile >= a.n_blocks) return;                             // (the whole block)
  const int lane = threadIdx.x & 63, l32 = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  extern __shared__ __align__(16) char smem[];
  char *stage = smem + wave * BS::BYTES;
  WG wg;
  wg.buf = reinterpret_cast<f32x4 (*)[WG::GF][64]>(smem + NW * BS::BYTES);
  wg.wave = wave; wg.lane = lane;

  // this wave's tile: waves past the last tile take the last one and store nothing (they still
  // meet the barriers, and their mask reads stay inside the arrays)
  const int64_t n_wt = KIND == KIND_EDGE ? a.n_tiles : (a.n_rows + 31) / 32;
  int64_t wt = tile * NW + wave;
  const bool none = wt >= n_wt;
  if (none) wt = n_wt - 1;
  int64_t row0;
  int n_valid;
  if constexpr (KIND == KIND_EDGE) {
    row0 = a.tile_ptr[wt];
    n_valid = none ? 0 : a.tile_ptr[wt + 1] - (int)row0;
  } else {
    row0 = wt * 32;
    const int64_t left = a.n_rows - row0;
    n_valid = none ? 0 : (left < 32 ? (int)left : 32);
  }
  int64_t row = row0 + l32;
  if (row >= a.n_rows) row = a.n_rows - 1;                    // clamp loads; stores are guarded
  int drow = (int)row;                                        // the row of dy this lane's row reads: itself, or its receiver
  if constexpr (KIND == KIND_EDGE) drow = a.in_dst[row];
  else if (a.dy_index) drow = a.dy_index[row];
  [[maybe_unused]] int fold_rem = 0, fold_dsel = -1;          // FOLD: edges after this one with its receiver; row of the total
  if constexpr (FOLD) {
    const bool valid = l32 < n_valid;
    const int up = __shfl_up(drow, 1);                        // lane 32 reads lane 31, but is a head anyway
    const bool head = valid && (l32 == 0 || up != drow);
    const uint64_t heads = ((uint64_t)(uint32_t)__ballot(head)) | ((uint64_t)1 << n_valid);
    fold_rem = valid ? __builtin_ctzll(heads >> (l32 + 1)) : 0;
    fold_dsel = head ? drow : -1;
  }
  [[maybe_unused]] int recv_dsel = -1;                        // NODE: this lane's row if it has in-edges
  if constexpr (KIND == KIND_NODE) recv_dsel = (l32 < n_valid && a.agg_src[row] >= 0) ? (int)row : -1;
  // mask bits of y (low half) and z1 (high half) of this lane's row, per 32-feature block
  uint32_t yz[MB];
#pragma unroll
  for (int nb = 0; nb < MB; ++nb) {
    uint32_t y = 0xffffu;
    if constexpr (!GIVEN) y = a.ymask[((size_t)wt * MB + nb) * 64 + lane];
    const uint32_t z = a.z1mask[((size_t)wt * MB + nb) * 64 + lane];
    yz[nb] = y | (z << 16);
  }

  // ---------------- dz2^T = dy^T * [y^T > 0], stored and kept as operand slabs.
  // The tile's dy rows are read as whole 64-byte pieces (four lanes per row, sixteen rows per
  // instruction: read with lane = row directly, every load instruction would touch 64 different
  // cache lines for 8 bytes each) and turned into the accumulator layout (lane = row) through the
  // wave's staging buffer. All of it is requested first and transposed before the first store: a
  // wait for a load that follows stores also waits for those stores to be acknowledged (one
  // counter, in order), which would put a memory round trip into every block.
  bf16x8 dz2s[MB][QB];
  {
    bf16x4 dyq[MB][4];
    {
      f32x4 raw[MB][32 / BS::RPI];
#pragma unroll
      for (int k = 0; k < 32 / BS::RPI; ++k) {
        const int src = __shfl(drow, k * BS::RPI + lane / BS::LPR);
        const char *p = (const char *)((const T *)a.dy + (size_t)src * H) + (lane % BS::LPR) * 16;
#pragma unroll
        for (int nb = 0; nb < MB; ++nb) raw[nb][k] = *(const f32x4 *)(p + 64 * nb);
      }
#pragma unroll
      for (int nb = 0; nb < MB; ++nb) {
#pragma unroll
        for (int k = 0; k < 32 / BS::RPI; ++k)
          *(f32x4 *)(stage + (k * BS::RPI + lane / BS::LPR) * BS::RS + (lane % BS::LPR) * 16) = raw[nb][k];
        wave_lds_fence();
#pragma unroll
        for (int q = 0; q < 4; ++q) dyq[nb][q] = *(const bf16x4 *)(stage + l32 * BS::RS + 16 * q + 8 * g);
        wave_lds_fence();
      }
    }
#pragma unroll
    for (int nb = 0; nb < MB; ++nb) {
      f32x16 d;
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int j = 0; j < 4; ++j) d[4 * q + j] = (yz[nb] >> (4 * q + j)) & 1u ? (float)dyq[nb][q][j] : 0.f;
      if constexpr (!GIVEN) store_block_via_lds<T, H>((T *)a.dz2, row0, n_valid, nb, lane, d, stage);
#pragma unroll
      for (int q = 0; q < QB; ++q) dz2s[nb][q] = acc_slab<T>(d, q);
    }
  }

  // ---------------- dz1^T = (W2 dz2^T) * [z1^T > 0]: unit mb = the W2^T fragments of block mb
  bf16x8 dz1s[MB][QB];
  {
    const bf16x8 *W2b = (const bf16x8 *)a.W2bt + lane;
    auto idx_from = [&](int u0) { return [=](int u, int j) { return j * MB + u0 + u; }; };
    wg.begin(W2b, idx_from(0));
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int g0 = mb / UG * UG, u = mb % UG;
      if (u == 0 && g0 + UG < MB) wg.fetch(W2b, idx_from(g0 + UG));
      f32x16 d;
#pragma unroll
      for (int r = 0; r < 16; ++r) d[r] = 0.f;
#pragma unroll
      for (int nb = 0; nb < MB; ++nb)
#pragma unroll
        for (int q = 0; q < QB; ++q) d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wg.get(u, nb * QB + q), dz2s[nb][q], d, 0, 0, 0);
      if (u == UG - 1) wg.next(g0 + UG < MB);
#pragma unroll
      for (int r = 0; r < 16; ++r) d[r] = (yz[mb] >> (16 + r)) & 1u ? d[r] : 0.f;
      store_block_via_lds<T, H>((T *)a.dz1, row0, n_valid, mb, lane, d, stage);
#pragma unroll
      for (int q = 0; q < QB; ++q) dz1s[mb][q] = acc_slab<T>(d, q);
    }
  }

  // ---------------- dx^T = W1 dz1^T over the first 2H input columns (the h-wide parts): unit kb =
  // the W1^T fragments of the 32-column block kb of [part a | part b]
  if constexpr (KIND != KIND_EMBED) {
    const bf16x8 *W1b = (const bf16x8 *)a.W1bt + lane;
    constexpr int KB = 2 * MB;
    auto idx_from = [&](int u0) { return [=](int u, int j) { return j * KB + u0 + u; }; };
    wg.begin(W1b, idx_from(0));
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
      const int g0 = kb / UG * UG, u = kb % UG;
      if (u == 0 && g0 + UG < KB) wg.fetch(W1b, idx_from(g0 + UG));
      f32x16 d;
#pragma unroll
      for (int r = 0; r < 16; ++r) d[r] = 0.f;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int q = 0; q < QB; ++q) d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wg.get(u, mb * QB + q), dz1s[mb][q], d, 0, 0, 0);
      if (u == UG - 1) wg.next(g0 + UG < KB);
      if (FOLD && kb >= MB) {
        // segmented suffix sum across the lanes of each receiver's run (see edge_tile_sum)
#pragma unroll
        for (int dd = 1; dd < 32; dd <<= 1) {
          if (__any(fold_rem >= dd)) {
            const float takef = fold_rem >= dd ? 1.f : 0.f;
            const int from = ((lane + dd) & 63) << 2;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const float v = d[r];
              const float t = dd == 1 ? __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x130, 0xf, 0xf, false))
                                      : __int_as_float(__builtin_amdgcn_ds_bpermute(from, __float_as_int(v)));
              d[r] = fmaf(t, takef, v);
            }
          }
        }
        store_block_rows_via_lds<T, H>((T *)a.dx_b, fold_dsel, kb % MB, lane, d, stage);
      } else if (KIND == KIND_NODE && kb >= MB) {
        store_block_rows_via_lds<T, H>((T *)a.dx_b, recv_dsel, kb % MB, lane, d, stage);
      } else {
        store_block_via_lds<T, H>((T *)(kb < MB ? a.dx_a : a.dx_b), row0, n_valid, kb % MB, lane, d, stage);
      }
    }
  }
}
