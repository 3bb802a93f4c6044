// Register-stationary variant of the fused two-layer MLP in bf16 (edge and node kinds):
// persistent blocks of H / 32 waves, wave w owning output features [32w, 32w + 32) of both
// layers. Its slices of W1 (2H/16 + 1 fragments) and W2 (H/16 fragments) stay in registers for
// the whole kernel, so the steady state moves no weights at all; what the waves of a block share
// instead is the input: a tile of 32 rows is gathered once per block into LDS and read by all
// its waves as MFMA operands, and layer 1's output is exchanged through LDS in operand fragment
// order. Used for H = 256, where the fragment-ordered weights (about 400 KB) fit neither LDS nor
// one wave's registers: one block of 8 waves per CU (a few W2 fragments are parked in LDS, the
// registers do not hold them all). The template also covers H = 128 (blocks of 4 waves, three
// per CU) and H = 64, but there the LDS-resident-weights kernel, whose waves run their tiles
// without block barriers, measured faster.
//
// The gather uses the loads that write LDS directly (16 bytes per lane, no registers in between;
// lane i of an instruction fills bytes [16 i, 16 i + 16) of a 1 KB destination): one instruction
// fetches 1024 / (2H) whole row parts, each lane one 16-byte piece, so global reads are whole rows.
// Which piece a lane fetches is permuted per row -- slot j of row r holds piece j ^ (r % 16) --
// which makes the operand reads (32 rows x the same piece) bank-conflict free without padding.
// The loads of tile t+2 are issued at the end of tile t into the buffer tile t just vacated and
// are awaited at the end of tile t+1: a whole tile of compute hides their latency. Row indices
// are requested one tile earlier still.
//
// Per tile (two block barriers):
//   layer 1: z1[32w.., rows] = W1[:, 32w..]^T x^T            2H/16 (+1) MFMAs per wave, x from LDS
//   ReLU, bf16, own two fragments -> zbuf; barrier
//   layer 2: y[32w.., rows] = W2[:, 32w..]^T relu(z1)^T       H/16 MFMAs per wave, z from LDS
//   epilogue on the wave's 32 features: NODE ReLU; EDGE ReLU + per-receiver sum across lanes;
//   rows -> staging buffer; wait for tile t+1's rows; barrier
//   whole rows stored, 16 bytes per lane; loads of tile t+2 issued
#pragma once
#include "mlp2.hip.h"

// 16 bytes per lane from global memory straight into LDS: lane i's piece lands at LDS byte
// lds_base + 16 i (lds_base uniform across the wave). Written as inline assembly on purpose:
// the compiler makes every later LDS access wait for its own LDS-direct loads, whichever
// buffer they target, which would serialise the prefetch with the compute it is meant to
// overlap. Whoever reads the destination must wait for vmcnt(0) and a barrier first.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void lds_direct_load16(const void *g, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_base)
               : "memory", "m0");
}
#pragma clang diagnostic pop
__device__ __forceinline__ unsigned lds_address(const void *p) {
  return (unsigned)(uintptr_t)(const __attribute__((address_space(3))) char *)p;
}

template <int H, int KIND>
struct RTile {
  static constexpr int MB = H / 32, NT = 64 * MB;                          // waves, threads per block
  static constexpr int ROWB = H * 2;                                       // bytes of one H-wide row part
  static constexpr int LPR = ROWB / 16;                                    // 16-byte pieces per row part
  static constexpr int RPI = 64 / LPR;                                     // row parts per load instruction
  static constexpr int SWM = LPR < 16 ? LPR - 1 : 15;                      // slot = piece ^ (row & SWM)
  static constexpr int XPART = 32 * ROWB;                                  // one H-wide part of 32 rows
  static constexpr int XBUF = 2 * XPART + (KIND == KIND_EDGE ? 1024 : 0);  // + raw fp32 edge attributes
  static constexpr int NC2 = H / 16;                                       // chunks of layer 2
  static constexpr int ZBUF = NC2 * 1024;                                  // chunks x 64 lanes x 16 bytes
  static constexpr int SROW = ROWB + 16, SBUF = 32 * SROW;                 // output staging, padded rows
  static constexpr int NC2L = H < 256 ? 0 : (KIND == KIND_EDGE ? 7 : 6);   // W2 fragments per wave kept in LDS
  static constexpr int W2L = MB * NC2L * 1024;
  static constexpr int BIAS = 2 * H * 4;
  static constexpr int BYTES = 2 * XBUF + ZBUF + SBUF + 256 + BIAS + W2L;  // + receiver rows, biases, W2 part
  static constexpr int WAVES_PER_SIMD = H == 256 ? 2 : (H == 128 ? 3 : 4); // occupancy the registers allow
};

// Rows of one tile: EDGE tiles are the packer's edge tiles, NODE tiles are 32 consecutive nodes.
struct RTileRows {
  int64_t r0;   // first row
  int nv;       // rows in the tile (1..32)
};
template <int KIND>
__device__ __forceinline__ RTileRows rtile_rows(const Mlp2Args &a, int64_t wt) {
  RTileRows t;
  if constexpr (KIND == KIND_EDGE) {
    // wt is uniform: read the tile table through the scalar unit (the constant address space; the
    // table is never written on the device). As an ordinary load it would be a vector load whose
    // result is needed in scalar registers at once, and the wait for it also waits for every row
    // prefetch issued just before.
    typedef const __attribute__((address_space(4))) int32_t *cptr;
    cptr tp = (cptr)(uintptr_t)a.tile_ptr;
    t.r0 = tp[wt];
    t.nv = tp[wt + 1] - (int)t.r0;
  } else {
    t.r0 = wt * 32;
    const int64_t left = a.n_rows - t.r0;
    t.nv = left < 32 ? (int)left : 32;
  }
  return t;
}

// What this lane fetches for a tile: a block issues H / 8 load instructions per tile, four per
// wave; instruction q = 4w + j covers row parts q * RPI .. of the tile (the first H / 16
// instructions the sender / node-state rows, the others the receiver / received-sum rows), and
// wave 0 also fetches the edge attributes. src[j] is the global row the lane reads for
// instruction j (rows past the tile's last repeat it and are never stored; NODE: the node's entry
// of agg_src, which must be given: -1 = zeros in place of its received sum). Nothing here branches
// on a loaded value, so the index loads can stay in flight until the rows are fetched a tile later.
struct RFetch {
  int src[4];
};
template <int H, int KIND>
__device__ __forceinline__ RFetch rtile_index(const Mlp2Args &a, const RTileRows &t, int w, int lane) {
  using R = RTile<H, KIND>;
  RFetch f;
  const int32_t *ip = w < R::MB / 2 ? a.in_src : a.in_dst;     // EDGE: first half senders, second half receivers
  int lq = lane / R::LPR;                                       // (opaque: recomputed per call, not four registers
  asm volatile("" : "+v"(lq));                                  //  of per-instruction row numbers kept across the loop)
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int r = R::RPI * ((4 * w + j) % (H / 16)) + lq;
    const int64_t row = t.r0 + (r < t.nv ? r : t.nv - 1);
    if constexpr (KIND == KIND_EDGE) f.src[j] = ip[row];
    else f.src[j] = a.agg_src[row];   // (requested by every wave, whichever part it fetches: a load under a
                                      //  condition would be waited for on the spot, behind the row prefetch)
  }
  return f;
}
template <int H, int KIND>
__device__ __forceinline__ void rtile_fetch(const Mlp2Args &a, const RTileRows &t, const RFetch &f, int w, int lane,
                                            char *xbuf) {
  using R = RTile<H, KIND>;
  const bf16_t *base = (KIND == KIND_NODE && w >= R::MB / 2) ? (const bf16_t *)a.agg : (const bf16_t *)a.h;
  int lv = lane;
  asm volatile("" : "+v"(lv));
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int q = 4 * w + j, r = R::RPI * (q % (H / 16)) + lv / R::LPR;
    const int piece = (lv % R::LPR) ^ (r & R::SWM);
    int64_t srow = f.src[j];
    if constexpr (KIND == KIND_NODE) {
      if (w < R::MB / 2) srow = t.r0 + (r < t.nv ? r : t.nv - 1);   // the node's own state
    }
    const bf16_t *rowp = srow < 0 ? (const bf16_t *)a.zero_row : base + (size_t)srow * H;
    lds_direct_load16(rowp + piece * 8, __builtin_amdgcn_readfirstlane(lds_address(xbuf) + q * 1024));
  }
  if constexpr (KIND == KIND_EDGE) {
    if (w == 0) {                                               // 32 rows x 32 bytes of raw fp32 attributes
      const int r = lane >> 1, half = lane & 1;
      const int64_t erow = t.r0 + (r < t.nv ? r : t.nv - 1);
      const void *g = 4 * half < a.De ? (const void *)(a.edge_feat + (size_t)erow * a.De + 4 * half)
                                      : (const void *)a.zero_row;
      lds_direct_load16(g, __builtin_amdgcn_readfirstlane(lds_address(xbuf) + 2 * R::XPART));
    }
  }
}

// SAVE: also keeps the forward for the backward pass (a.z1, a.z1mask, a.ymask; see Mlp2Args). relu(z1) leaves
// as whole rows through the input buffer of the tile itself, which is idle between the end of
// layer 1 and the prefetch of the tile after next: after the first barrier every wave writes its
// 32 features of all rows there, after the second barrier wave w reads rows 4w .. 4w+3 back and
// stores them -- from the 4 KB of the buffer that only its own prefetch loads write, so no wave
// waits for another. Row r sits at 4096 (r / 4) + 64 ((r / 4) % 4) + 528 (r % 4): 16-byte aligned,
// and the 8-byte writes of 32 rows fall on 16 different bank groups.
template <int H, int KIND, bool SAVE>
__global__ __launch_bounds__((RTile<H, KIND>::NT), (RTile<H, KIND>::WAVES_PER_SIMD)) void mlp2r_kernel(const Mlp2Args a) {
  using T = bf16_t;
  using R = RTile<H, KIND>;
  constexpr int MB = R::MB, HS = H / 16, NT = R::NT;
  constexpr int NS1 = 2 * HS + (KIND == KIND_EDGE ? 1 : 0), NC2 = R::NC2;
  static_assert(KIND == KIND_EDGE || KIND == KIND_NODE, "edge and node MLPs only");
  static_assert(H == 64 || H == 128 || H == 256, "hidden width");
  extern __shared__ __align__(16) char smem[];
  char *zbuf = smem + 2 * R::XBUF;
  char *sbuf = zbuf + R::ZBUF;
  int *drow = (int *)(sbuf + R::SBUF);                         // EDGE: destination row of each staged row
  float(*b1l)[2][16] = (float(*)[2][16])(sbuf + R::SBUF + 256), (*b2l)[2][16] = b1l + MB;

  const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, g = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);      // (uniform: what derives from it stays in scalar registers)
  const int nbx = gridDim.x / 8, xcd = blockIdx.x % 8, lid = blockIdx.x / 8;
  const int64_t n_wt = KIND == KIND_EDGE ? a.n_tiles : (a.n_rows + 31) / 32;
  const int64_t per_xcd = (n_wt + 7) / 8;
  const int64_t t_begin = xcd * per_xcd;
  const int64_t t_end = (t_begin + per_xcd) < n_wt ? (t_begin + per_xcd) : n_wt;
  int64_t wt = t_begin + lid;
  if (wt >= t_end) return;                                     // the whole block leaves together

  // first two tiles' rows, third tile's indices
  RTileRows cur = rtile_rows<KIND>(a, wt);
  RTileRows nxt = cur;
  rtile_fetch<H, KIND>(a, cur, rtile_index<H, KIND>(a, cur, w, lane), w, lane, smem);
  if (wt + nbx < t_end) {
    nxt = rtile_rows<KIND>(a, wt + nbx);
    rtile_fetch<H, KIND>(a, nxt, rtile_index<H, KIND>(a, nxt, w, lane), w, lane, smem + R::XBUF);
  }
  RTileRows nn = nxt;
  RFetch fn;
  if (wt + 2 * nbx < t_end) {
    nn = rtile_rows<KIND>(a, wt + 2 * nbx);
    fn = rtile_index<H, KIND>(a, nn, w, lane);
  }
  // this wave's weight slices, loaded once, and the biases in accumulator order (parked in LDS:
  // the weight slices leave few registers)
  constexpr int NC2R = NC2 - R::NC2L;                         // W2 fragments in registers; the rest in LDS
  bf16x8 W1r[NS1], W2r[NC2R];
  [[maybe_unused]] bf16x8 *W2l = (bf16x8 *)((char *)(b2l + MB) + w * R::NC2L * 1024) + lane;   // [NC2L][64] of this wave
  {
    const bf16x8 *s1 = (const bf16x8 *)a.W1s + w * 64 + lane, *s2 = (const bf16x8 *)a.W2s + w * 64 + lane;
#pragma unroll
    for (int s = 0; s < NS1; ++s) W1r[s] = s1[(size_t)s * MB * 64];
#pragma unroll
    for (int c = 0; c < NC2R; ++c) W2r[c] = s2[(size_t)c * MB * 64];
#pragma unroll
    for (int c = NC2R; c < NC2; ++c) W2l[(c - NC2R) * 64] = s2[(size_t)c * MB * 64];
  }
  // This lane's operand piece 2k + g of row l32 sits in slot (2k + g) ^ (l32 & SWM) of its row part,
  // i.e. at byte xrow + ((k ^ xk) << 5); pieces 16.. add 256. (Recomputed per read: two VALU
  // instructions are cheaper here than eight more live registers.)
  const int xk = (l32 & R::SWM) >> 1;
  const int xrow = l32 * R::ROWB + (((l32 ^ g) & 1) << 4);
  if (tid < MB * 32) {
    b1l[tid / 32][(tid / 16) % 2][tid % 16] = a.b1[32 * (tid / 32) + acc_row(tid % 16, (tid / 16) % 2)];
    b2l[tid / 32][(tid / 16) % 2][tid % 16] = a.b2[32 * (tid / 32) + acc_row(tid % 16, (tid / 16) % 2)];
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);                          // vmcnt(0): both tiles' rows are in LDS
  __syncthreads();

  int buf = 0;
  for (; wt < t_end; wt += nbx) {
    const char *xb = smem + buf * R::XBUF;
    asm volatile("" ::: "memory");
    [[maybe_unused]] EdgeTileMeta m;
    if constexpr (KIND == KIND_EDGE) m = load_edge_meta(a.in_dst, a.n_rows, cur.r0, cur.nv, l32);
    // ---------------- layer 1: this wave's 32 features x the tile's rows (each operand is read
    // from LDS ahead of the MFMA that uses it)
    f32x16 acc = *(const f32x16 *)&b1l[w][g][0];
    {
      int xk_t = xk;
      asm volatile("" : "+v"(xk_t));                             // keeps the eight offsets out of registers
      auto xread = [&](int s) {
        const int k = s % HS;                                     // slab inside its row part
        return *(const bf16x8 *)(xb + (s / HS) * R::XPART + (k >> 3) * 256 + xrow + (((k & 7) ^ xk_t) << 5));
      };
      constexpr int RA = KIND == KIND_NODE ? 3 : 2;             // operands read ahead of their MFMA
      bf16x8 xq[RA + 1];
#pragma unroll
      for (int i = 0; i < RA; ++i) xq[i] = xread(i);
#pragma unroll
      for (int s = 0; s < 2 * HS; ++s) {
        if (s + RA < 2 * HS) xq[(s + RA) % (RA + 1)] = xread(s + RA);
        __builtin_amdgcn_sched_barrier(0);                      // keep the read ahead of the MFMA it follows
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(W1r[s], xq[s % (RA + 1)], acc, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      if constexpr (KIND == KIND_EDGE) {
        const float *xe = (const float *)(xb + 2 * R::XPART + l32 * 32);
        TailRaw<8> raw;
        raw.q[0] = *(const f32x4 *)xe;
        raw.q[1] = *(const f32x4 *)(xe + 4);
        const bf16x8 xt = g == 0 ? tail_to_operand<T>(raw) : Operand<bf16_t>::zero();
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(W1r[2 * HS], xt, acc, 0, 0, 0);
      }
    }
#pragma unroll
    for (int q = 0; q < 2; ++q)
      *(bf16x8 *)(zbuf + ((2 * w + q) * 64 + lane) * 16) = relu_operand<T>(acc, q);
    if constexpr (SAVE) {
      int lv = lane;
      asm volatile("" : "+v"(lv));
      a.z1mask[((size_t)wt * MB + w) * 64 + lv] = lane_mask_bits(acc);
    }
    __syncthreads();
    if constexpr (SAVE) {
      static_assert(!SAVE || H == 256, "the staging layout below is laid out for eight waves");
      typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
      // (addresses from an opaque copy of the lane id: computed here in every tile instead of
      // living in registers across the loop, which has none to spare)
      int lv = lane;
      asm volatile("" : "+v"(lv));
      const int r_ = lv & 31, g_ = lv >> 5;
      char *zrow = smem + buf * R::XBUF + 4096 * (r_ >> 2) + 64 * ((r_ >> 2) & 3) + 528 * (r_ & 3) + (32 * w + 4 * g_) * 2;
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const u32x4 z = __builtin_bit_cast(u32x4, relu_operand<T>(acc, q));   // features 16 q + 4 g + {0..3}, + 8
        *(u32x2 *)(zrow + 32 * q) = u32x2{z[0], z[1]};
        *(u32x2 *)(zrow + 32 * q + 16) = u32x2{z[2], z[3]};
      }
    }
    // ---------------- layer 2
    acc = *(const f32x16 *)&b2l[w][g][0];
    {
      const bf16x8 *zr = (const bf16x8 *)zbuf + lane;
      // z fragments are read two chunks ahead, the W2 fragments parked in LDS one chunk ahead
      bf16x8 zq[3], wl = W2r[0];
      zq[0] = zr[0];
      zq[1] = zr[64];
#pragma unroll
      for (int c = 0; c < NC2; ++c) {
        if (c + 2 < NC2) zq[(c + 2) % 3] = zr[(c + 2) * 64];
        const bf16x8 wf = c < NC2R ? W2r[c < NC2R ? c : 0] : wl;
        if constexpr (R::NC2L > 0) {
          if (c + 1 >= NC2R && c + 1 < NC2) wl = W2l[(c + 1 - NC2R) * 64];
        }
        __builtin_amdgcn_sched_barrier(0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, zq[c % 3], acc, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if constexpr (SAVE) {
      __builtin_amdgcn_sched_barrier(0);
      int lv = lane;
      asm volatile("" : "+v"(lv));
      a.ymask[((size_t)wt * MB + w) * 64 + lv] = lane_mask_bits(acc);
      __builtin_amdgcn_sched_barrier(0);
    }
    // ---------------- epilogue on this wave's 32 features
    T *out = (T *)a.out;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = relu_f32(acc[r]);
    if constexpr (KIND == KIND_EDGE) {
      const bool valid = l32 < cur.nv;
      const int up = __shfl_up(m.dst, 1);
      const bool head = valid && (l32 == 0 || up != m.dst);
      const uint64_t heads = ((uint64_t)(uint32_t)__ballot(head)) | ((uint64_t)1 << cur.nv);
      const int rem = valid ? __builtin_ctzll(heads >> (l32 + 1)) : 0;
#pragma unroll
      for (int d = 1; d < 32; d <<= 1) {                        // see edge_tile_sum
        if (__any(rem >= d)) {
          const float takef = rem >= d ? 1.f : 0.f;
          const int from = ((lane + d) & 63) << 2;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float v = acc[r];
            const float t = d == 1 ? __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x130, 0xf, 0xf, false))
                                   : __int_as_float(__builtin_amdgcn_ds_bpermute(from, __float_as_int(v)));
            acc[r] = fmaf(t, takef, v);
          }
        }
      }
      const bool ends_tile = l32 + rem == cur.nv - 1;
      const bool to_c0 = head && l32 == 0 && m.prev_d == m.dst;
      const bool to_c1 = head && !to_c0 && ends_tile && m.next_d == m.dst;
      if (w == 0 && g == 0) drow[l32] = (head && !to_c0 && !to_c1) ? m.dst : -1;
      if (to_c0 || to_c1) {
        float *cp = a.carry + ((size_t)wt * 2 + (to_c1 ? 1 : 0)) * H + 32 * w + 4 * g;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float v[4] = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
          store4<float>(cp + 8 * q, v);
        }
      }
    }
    {
      char *sp = sbuf + l32 * R::SROW + (32 * w + 4 * g) * 2;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float v[4] = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
        store4<T>((T *)(sp + 16 * q), v);
      }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                        // vmcnt(0): the next tile's rows are in LDS
    __syncthreads();
    {
      const int piece = tid % R::LPR, rr = tid / R::LPR;          // 16 rows per pass
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int r = rr + 16 * j;
        const f32x4 v = *(const f32x4 *)(sbuf + r * R::SROW + piece * 16);
        int64_t drw;
        if constexpr (KIND == KIND_EDGE) drw = drow[r];
        else drw = r < cur.nv ? cur.r0 + r : -1;
        if (drw >= 0) *(f32x4 *)((char *)(out + (size_t)drw * H) + piece * 16) = v;
      }
    }
    if constexpr (SAVE) {
      __builtin_amdgcn_sched_barrier(0);                         // (after the output rows: not interleaved with them)
      // this wave's four rows of relu(z1), from its own part of the tile's input buffer
      const char *zreg = smem + buf * R::XBUF + 4096 * w + 64 * (w & 3);
      int lv = lane;
      asm volatile("" : "+v"(lv));
      const int r_ = lv & 31, g_ = lv >> 5;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int j = 2 * i + g_, r = 4 * w + j;
        const f32x4 v = *(const f32x4 *)(zreg + 528 * j + 16 * r_);
        if (r < cur.nv) *(f32x4 *)((char *)((T *)a.z1 + (size_t)(cur.r0 + r) * H) + 16 * r_) = v;
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    // the buffer this tile used is free now: rows of the tile after next, indices one further
    if (wt + 2 * nbx < t_end) rtile_fetch<H, KIND>(a, nn, fn, w, lane, smem + buf * R::XBUF);
    cur = nxt;
    nxt = nn;
    if (wt + 3 * nbx < t_end) {
      nn = rtile_rows<KIND>(a, wt + 3 * nbx);
      fn = rtile_index<H, KIND>(a, nn, w, lane);
    }
    buf ^= 1;
  }
}
