// Backward of the fused two-layer ReLU MLPs from what the forward pass kept (Section 3.3.4: one
// back-propagation through the GNN of Section 3.4), bf16, for the batches whose forward kernels
// store the hidden activation relu(z1) [rows, H] (and, for the edge MLP, whose per-edge output y is
// never stored, the mask bits of y > 0). With them the backward needs no forward arithmetic at
// all and no gathered input rows:
//     dz2 = dy * [y > 0],  dz1 = (dz2 W2^T) * [z1 > 0],  dx = dz1 W1^T
// [y > 0] comes from the stored output (NODE: the next node states, EMBED: the first) or from the
// kept mask bits (EDGE), [z1 > 0] from the kept relu(z1). dz2 and dz1 are stored for the
// weight-gradient kernel, which reads z1 from the forward's copy. Everything is kept transposed
// (features x rows: lane = row, registers = features), each result already laid out as the next
// contraction's B operand, as in mlp2_bwd_kernel; the three live tiles of that kernel (z1, dz2,
// dz1) shrink to two, which lets eight waves share a compute unit at H = 256. The weights go
// through the same double-buffered LDS groups, fetched once per block of NW waves. A wave's tile
// is 32 consecutive rows; for EDGE it is an edge tile of the packer (at most 32 edges), because
// the kept mask bits are per tile and lane of the forward kernel. Those tiles are cut at receiver
// boundaries, so with FOLD (batches in which no receiver has more than 32 in-edges) the gradients
// w.r.t. h_receiver are summed per receiver across the lanes of the tile, as the forward sums the
// messages, and leave as one row per receiver instead of one per edge.
#pragma once
#include "mlp2_bwd.hip.h"

struct Mlp2BwdzArgs {
  int64_t n_rows, n_blocks;
  const void *W2bt, *W1bt;     // contraction over the weight's columns (see swizzle_chain)
  const void *dy;              // upstream gradient [N, H] bf16 (EDGE: indexed by receiver)
  const void *z1;              // relu(z1) [rows, H] bf16, kept by the forward
  const void *y;               // the forward's output [N, H] bf16 (NODE, EMBED)
  const uint16_t *ymask;       // EDGE: [n_tiles][H / 32][64] mask bits of y (see Mlp2Args)
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

template <int H, int KIND, bool FOLD>
__global__ __launch_bounds__((64 * BwdzShape<H>::NW)) void mlp2_bwdz_kernel(const Mlp2BwdzArgs a) {
  static_assert(!FOLD || KIND == KIND_EDGE, "only the edge MLP's receiver-side gradients are summed");
  using T = bf16_t;
  using S = BwdzShape<H>;
  constexpr int MB = S::MB, QB = S::QB, UF = S::UF, UG = S::UG, NW = S::NW;
  using WG = WeightGroupsN<UF, UG, NW>;
  const int64_t per_xcd = (a.n_blocks + 7) / 8;
  const int64_t tile = (int64_t)(blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (tile >= a.n_blocks) return;                             // (the whole block)
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l32 = lane & 31, g = lane >> 5;
  int64_t wt = tile * NW + wave;                              // this wave's tile
  int64_t row0;
  int n_valid;
  if constexpr (KIND == KIND_EDGE) {
    const bool none = wt >= a.n_tiles;                        // (waves past the last tile still meet the barriers)
    if (none) wt = a.n_tiles - 1;
    row0 = a.tile_ptr[wt];
    n_valid = none ? 0 : a.tile_ptr[wt + 1] - (int)row0;
  } else {
    row0 = wt * 32;
    const int64_t left = a.n_rows - row0;
    n_valid = left < 32 ? (left > 0 ? (int)left : 0) : 32;
  }
  int64_t row = row0 + l32;
  if (row >= a.n_rows) row = a.n_rows - 1;                    // clamp loads; stores are guarded
  extern __shared__ __align__(16) char smem[];
  char *stage = smem + wave * BlockStage<T>::BYTES;
  WG wg;
  wg.buf = reinterpret_cast<f32x4 (*)[WG::GF][64]>(smem + NW * BlockStage<T>::BYTES);
  wg.wave = wave; wg.lane = lane;

  // one 32-feature block of this lane's row of a row-major [rows, H] array, in accumulator order
  auto load_block = [&](const T *rowp, int nb, f32x16 &d) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float v[4];
      load4<T>(rowp + 32 * nb + 8 * q, v);
      d[4 * q] = v[0]; d[4 * q + 1] = v[1]; d[4 * q + 2] = v[2]; d[4 * q + 3] = v[3];
    }
  };

  // ---------------- dz2^T = dy^T * [y^T > 0], stored and kept as operand slabs
  bf16x8 dz2s[MB][QB];
  [[maybe_unused]] int fold_rem = 0, fold_dsel = -1;          // FOLD: edges after this one with its receiver; row of the total
  {
    int64_t drow = row;
    if constexpr (KIND == KIND_EDGE) drow = a.in_dst[row];
    if constexpr (FOLD) {
      const bool valid = l32 < n_valid;
      const int dst = (int)drow, up = __shfl_up(dst, 1);      // lane 32 reads lane 31, but is a head anyway
      const bool head = valid && (l32 == 0 || up != dst);
      const uint64_t heads = ((uint64_t)(uint32_t)__ballot(head)) | ((uint64_t)1 << n_valid);
      fold_rem = valid ? __builtin_ctzll(heads >> (l32 + 1)) : 0;
      fold_dsel = head ? dst : -1;
    }
    const T *dyrow = (const T *)a.dy + (size_t)drow * H + 4 * g;
    [[maybe_unused]] const T *yrow = KIND == KIND_EDGE ? nullptr : (const T *)a.y + (size_t)row * H + 4 * g;
    [[maybe_unused]] uint32_t ym[MB];
    if constexpr (KIND == KIND_EDGE) {
#pragma unroll
      for (int nb = 0; nb < MB; ++nb) ym[nb] = a.ymask[((size_t)wt * MB + nb) * 64 + lane];
    }
    f32x16 dyc, yc, dyn, yn;
    load_block(dyrow, 0, dyc);
    if constexpr (KIND != KIND_EDGE) load_block(yrow, 0, yc);
#pragma unroll
    for (int nb = 0; nb < MB; ++nb) {
      if (nb + 1 < MB) {
        load_block(dyrow, nb + 1, dyn);
        if constexpr (KIND != KIND_EDGE) load_block(yrow, nb + 1, yn);
      }
      f32x16 d;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if constexpr (KIND == KIND_EDGE) d[r] = (ym[nb] >> r) & 1u ? dyc[r] : 0.f;
        else d[r] = yc[r] > 0.f ? dyc[r] : 0.f;
      }
      store_block_via_lds<T, H>((T *)a.dz2, row0, n_valid, nb, lane, d, stage);
#pragma unroll
      for (int q = 0; q < QB; ++q) dz2s[nb][q] = acc_slab<T>(d, q);
      if (nb + 1 < MB) { dyc = dyn; yc = yn; }
    }
  }

  // ---------------- dz1^T = (W2 dz2^T) * [z1^T > 0]: unit mb = the W2^T fragments of block mb
  bf16x8 dz1s[MB][QB];
  {
    const bf16x8 *W2b = (const bf16x8 *)a.W2bt + lane;
    auto idx_from = [&](int u0) { return [=](int u, int j) { return j * MB + u0 + u; }; };
    const T *zrow = (const T *)a.z1 + (size_t)row * H + 4 * g;
    f32x16 zc, zn;
    load_block(zrow, 0, zc);
    wg.begin(W2b, idx_from(0));
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int g0 = mb / UG * UG, u = mb % UG;
      if (u == 0 && g0 + UG < MB) wg.fetch(W2b, idx_from(g0 + UG));
      if (mb + 1 < MB) load_block(zrow, mb + 1, zn);
      f32x16 d;
#pragma unroll
      for (int r = 0; r < 16; ++r) d[r] = 0.f;
#pragma unroll
      for (int nb = 0; nb < MB; ++nb)
#pragma unroll
        for (int q = 0; q < QB; ++q) d = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wg.get(u, nb * QB + q), dz2s[nb][q], d, 0, 0, 0);
      if (u == UG - 1) wg.next(g0 + UG < MB);
#pragma unroll
      for (int r = 0; r < 16; ++r) d[r] = zc[r] > 0.f ? d[r] : 0.f;
      store_block_via_lds<T, H>((T *)a.dz1, row0, n_valid, mb, lane, d, stage);
#pragma unroll
      for (int q = 0; q < QB; ++q) dz1s[mb][q] = acc_slab<T>(d, q);
      if (mb + 1 < MB) zc = zn;
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
      } else {
        store_block_via_lds<T, H>((T *)(kb < MB ? a.dx_a : a.dx_b), row0, n_valid, kb % MB, lane, d, stage);
      }
    }
  }
}
