// MFMA operand traits for gfx950: one "slab" is the 16 bytes of contraction-dimension data a
// lane feeds to the 32x32 matrix instruction(s): 8 bf16 (one v_mfma_f32_32x32x16_bf16) or 4 fp32
// (four v_mfma_f32_32x32x2_f32). In both cases lane l addresses matrix row/column l % 32 and
// lane group g = l / 32 supplies its own half of the slab's contraction indices.
//
// Accumulator layout of a 32x32 tile (16 fp32 per lane): register r of lane l holds
//   row  8 * (r / 4) + 4 * (l / 32) + (r % 4),   column  l % 32.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16_t;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <typename T>
struct Operand;

template <>
struct Operand<float> {
  static constexpr int V = 4;  // elements per lane per slab
  typedef f32x4 vec;
  static __device__ __forceinline__ void mma(const vec &a, const vec &b, f32x16 &c) {
#pragma unroll
    for (int j = 0; j < 4; ++j) c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[j], b[j], c, 0, 0, 0);
  }
  static __device__ __forceinline__ float from_float(float x) { return x; }
  static __device__ __forceinline__ float to_float(float x) { return x; }
  static __device__ __forceinline__ vec zero() { return vec{0.f, 0.f, 0.f, 0.f}; }
};

template <>
struct Operand<bf16_t> {
  static constexpr int V = 8;
  typedef bf16x8 vec;
  static __device__ __forceinline__ void mma(const vec &a, const vec &b, f32x16 &c) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ bf16_t from_float(float x) { return (bf16_t)x; }
  static __device__ __forceinline__ float to_float(bf16_t x) { return (float)x; }
  static __device__ __forceinline__ vec zero() {
    vec z;
#pragma unroll
    for (int j = 0; j < 8; ++j) z[j] = (bf16_t)0.0f;
    return z;
  }
};

// row of accumulator register r inside its 32x32 tile, for lane group g
__device__ __forceinline__ int acc_row(int r, int g) { return 8 * (r >> 2) + 4 * g + (r & 3); }

// ReLU + conversion of V consecutive accumulator registers (chunk q of a 32x32 tile) into one
// MFMA operand. For bf16 the values are converted first and the ReLU is taken on the packed
// pairs as 16-bit integers (a negative bf16 has its sign bit set, i.e. is a negative int16;
// max(x, 0) maps it -- and -0 -- to +0 and leaves non-negative values untouched): half the
// instructions of ReLU-then-convert.
// max(x, 0) as a single integer max on the bit pattern (a negative float is a negative int32;
// -0 becomes +0). fmaxf costs a second instruction that quiets a possible signalling NaN first.
__device__ __forceinline__ float relu_f32(float x) {
  const int b = __float_as_int(x);
  return __int_as_float(b > 0 ? b : 0);
}

template <typename T>
__device__ __forceinline__ typename Operand<T>::vec relu_operand(const f32x16 &acc, int q);
template <>
__device__ __forceinline__ f32x4 relu_operand<float>(const f32x16 &acc, int q) {
  f32x4 z;
#pragma unroll
  for (int j = 0; j < 4; ++j) z[j] = relu_f32(acc[4 * q + j]);
  return z;
}
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// Two floats -> two bf16 (round to nearest even), `lo` in bits 15..0, `hi` in bits 31..16. Written
// as a two-element vector conversion, which the compiler selects as a single v_cvt_pk_bf16_f32
// (element-wise conversions of longer vectors cost one instruction per element plus a byte
// permute per pair). Deliberately not inline assembly: the compiler does not see the registers
// an asm statement reads, and so would not insert the wait states the hardware needs between a
// matrix instruction and the first read of its result.
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned cvt_pk_bf16(float lo, float hi) {
  const f32x2 f = {lo, hi};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16x2));
}
__device__ __forceinline__ bf16x8 pack_bf16x8(float x0, float x1, float x2, float x3, float x4, float x5,
                                              float x6, float x7) {
  const u32x4 u = {cvt_pk_bf16(x0, x1), cvt_pk_bf16(x2, x3), cvt_pk_bf16(x4, x5), cvt_pk_bf16(x6, x7)};
  return __builtin_bit_cast(bf16x8, u);
}

template <>
__device__ __forceinline__ bf16x8 relu_operand<bf16_t>(const f32x16 &acc, int q) {
  const bf16x8 z = pack_bf16x8(acc[8 * q], acc[8 * q + 1], acc[8 * q + 2], acc[8 * q + 3], acc[8 * q + 4],
                               acc[8 * q + 5], acc[8 * q + 6], acc[8 * q + 7]);
  s16x8 s = __builtin_bit_cast(s16x8, z);
  const s16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
  s = __builtin_elementwise_max(s, zero);
  return __builtin_bit_cast(bf16x8, s);
}

// four consecutive features of one row, starting at feature f0, as floats
template <typename T>
__device__ __forceinline__ void load4(const T *p, float *v);
template <>
__device__ __forceinline__ void load4<float>(const float *p, float *v) {
  f32x4 x = *(const f32x4 *)p;
  v[0] = x[0]; v[1] = x[1]; v[2] = x[2]; v[3] = x[3];
}
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
template <>
__device__ __forceinline__ void load4<bf16_t>(const bf16_t *p, float *v) {
  bf16x4 x = *(const bf16x4 *)p;
#pragma unroll
  for (int j = 0; j < 4; ++j) v[j] = (float)x[j];
}
template <typename T>
__device__ __forceinline__ void store4(T *p, const float *v);
template <>
__device__ __forceinline__ void store4<float>(float *p, const float *v) {
  *(f32x4 *)p = f32x4{v[0], v[1], v[2], v[3]};
}
template <>
__device__ __forceinline__ void store4<bf16_t>(bf16_t *p, const float *v) {
  typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
  *(u32x2 *)p = u32x2{cvt_pk_bf16(v[0], v[1]), cvt_pk_bf16(v[2], v[3])};
}

// four consecutive features of one row in their stored form
template <typename T>
struct Quad;
template <>
struct Quad<float> {
  typedef f32x4 type;
  static __device__ __forceinline__ type pack(const float *v) { return f32x4{v[0], v[1], v[2], v[3]}; }
};
template <>
struct Quad<bf16_t> {
  typedef unsigned type __attribute__((ext_vector_type(2)));
  static __device__ __forceinline__ type pack(const float *v) {
    return type{cvt_pk_bf16(v[0], v[1]), cvt_pk_bf16(v[2], v[3])};
  }
};

// Writes a features x rows accumulator tile (feature block fb) to a row-major [rows, H] array:
// lane = row, register quads = four consecutive features.
template <typename TO, int H>
__device__ __forceinline__ void store_tile_rows(TO *base, int64_t row, bool valid, int fb, int g,
                                                const f32x16 &acc) {
  if (!valid) return;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    float v[4] = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
    store4<TO>(base + (size_t)row * H + 32 * fb + 8 * q + 4 * g, v);
  }
}

// Same with ReLU applied on the way out.
template <typename TO, int H>
__device__ __forceinline__ void store_tile_rows_relu(TO *base, int64_t row, bool valid, int fb, int g,
                                                     const f32x16 &acc) {
  if (!valid) return;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    float v[4] = {relu_f32(acc[4 * q]), relu_f32(acc[4 * q + 1]), relu_f32(acc[4 * q + 2]),
                  relu_f32(acc[4 * q + 3])};
    store4<TO>(base + (size_t)row * H + 32 * fb + 8 * q + 4 * g, v);
  }
}

// Row-major store of a features x rows accumulator set (lane = row of a 32-row wave tile) through
// a wave-private LDS staging buffer, so that every global store instruction writes whole rows:
// a lane holds its own row, and storing from that layout directly would touch 32 different rows
// (cache lines) with every instruction. The tile goes through the buffer RP rows at a time: the
// lanes owning those rows write their register quads (padded row stride, bank-conflict free),
// then all 64 lanes read the rows back 16 bytes per lane, H * sizeof(T) / 16 lanes per row, and
// store them. row_dst(r) gives the destination of tile row r (nullptr: skip); it is called by all
// lanes together, so it may use cross-lane operations.
template <typename T, int H>
struct RowStage {
  static constexpr int RS = H * (int)sizeof(T) + 16;                  // padded row stride, bytes
  static constexpr int RP = H * (int)sizeof(T) >= 1024 ? 8 : 16;      // rows per pass
  static constexpr int BYTES = RP * RS;                               // per wave
  static constexpr int LPR = H * (int)sizeof(T) / 16;                 // lanes per row on the way out
  static constexpr int RPI = 64 / LPR;                                // rows per store instruction
};

__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <typename T, int H, bool RELU, typename RowDst>
__device__ __forceinline__ void store_rows_via_lds(const f32x16 (&acc)[H / 32], char *stage, int lane,
                                                   RowDst row_dst) {
  using S = RowStage<T, H>;
  using Q = typename Quad<T>::type;
  const int l32 = lane & 31, g = lane >> 5;
  // converted once, before the passes (inside a pass only the lanes of its rows are active, and
  // every pass would repeat the conversions)
  Q quad[H / 32][4];
#pragma unroll
  for (int nb = 0; nb < H / 32; ++nb)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float v[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = RELU ? relu_f32(acc[nb][4 * q + j]) : acc[nb][4 * q + j];
      quad[nb][q] = Quad<T>::pack(v);
    }
#pragma unroll
  for (int p = 0; p < 32 / S::RP; ++p) {
    if (l32 / S::RP == p) {
      char *wp = stage + (l32 % S::RP) * S::RS + 4 * g * (int)sizeof(T);
#pragma unroll
      for (int nb = 0; nb < H / 32; ++nb)
#pragma unroll
        for (int q = 0; q < 4; ++q) *(Q *)(wp + (32 * nb + 8 * q) * (int)sizeof(T)) = quad[nb][q];
    }
    wave_lds_fence();
#pragma unroll
    for (int k = 0; k < S::RP / S::RPI; ++k) {
      const int rr = k * S::RPI + lane / S::LPR;                      // row inside the pass
      const f32x4 v = *(const f32x4 *)(stage + rr * S::RS + (lane % S::LPR) * 16);
      T *dst = row_dst(p * S::RP + rr);
      if (dst) *(f32x4 *)((char *)dst + (lane % S::LPR) * 16) = v;
    }
    wave_lds_fence();
  }
}

// One 32-feature block of a features x rows accumulator tile (lane = row) to a row-major
// [rows, H] array, through a wave-private LDS buffer: the block's 32 rows x 32 elements are
// written as register quads and read back 16 bytes per lane, so a store instruction covers
// 64 / (32 * sizeof(TO) / 16) rows with one contiguous 32-element piece each, instead of 32 rows
// with 4 elements each. Rows row0 .. row0 + n_valid - 1 are stored. stage: BlockStage<TO>::BYTES.
template <typename TO>
struct BlockStage {
  static constexpr int RB = 32 * (int)sizeof(TO);        // bytes of a row's piece
  static constexpr int RS = RB + 16;                     // padded
  static constexpr int BYTES = 32 * RS;
  static constexpr int LPR = RB / 16, RPI = 64 / LPR;    // lanes per row, rows per instruction
};
template <typename TO, int H>
__device__ __forceinline__ void store_block_via_lds(TO *base, int64_t row0, int n_valid, int fb, int lane,
                                                    const f32x16 &d, char *stage) {
  using S = BlockStage<TO>;
  const int l32 = lane & 31, g = lane >> 5;
  char *wp = stage + l32 * S::RS + 4 * g * (int)sizeof(TO);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    float v[4] = {d[4 * q], d[4 * q + 1], d[4 * q + 2], d[4 * q + 3]};
    store4<TO>((TO *)(wp + 8 * q * (int)sizeof(TO)), v);
  }
  wave_lds_fence();
#pragma unroll
  for (int k = 0; k < 32 / S::RPI; ++k) {
    const int r = k * S::RPI + lane / S::LPR;
    const f32x4 v = *(const f32x4 *)(stage + r * S::RS + (lane % S::LPR) * 16);
    if (r < n_valid)
      *(f32x4 *)((char *)(base + (size_t)(row0 + r) * H + 32 * fb) + (lane % S::LPR) * 16) = v;
  }
  wave_lds_fence();
}

// The same for a block already held as two bf16 operand fragments (relu_operand of accumulator
// registers 0..7 and 8..15: features 4 g + {0..3} + 8 k, k = 0..3, of the lane's row).
template <int H>
__device__ __forceinline__ void store_block_fragments_via_lds(bf16_t *base, int64_t row0, int n_valid, int fb, int lane,
                                                              const bf16x8 &f0, const bf16x8 &f1, char *stage) {
  using S = BlockStage<bf16_t>;
  typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
  const int l32 = lane & 31, g = lane >> 5;
  char *wp = stage + l32 * S::RS + 4 * g * 2;
  const u32x4 z0 = __builtin_bit_cast(u32x4, f0), z1 = __builtin_bit_cast(u32x4, f1);
  *(u32x2 *)(wp) = u32x2{z0[0], z0[1]};
  *(u32x2 *)(wp + 16) = u32x2{z0[2], z0[3]};
  *(u32x2 *)(wp + 32) = u32x2{z1[0], z1[1]};
  *(u32x2 *)(wp + 48) = u32x2{z1[2], z1[3]};
  wave_lds_fence();
#pragma unroll
  for (int k = 0; k < 32 / S::RPI; ++k) {
    const int r = k * S::RPI + lane / S::LPR;
    const f32x4 v = *(const f32x4 *)(stage + r * S::RS + (lane % S::LPR) * 16);
    if (r < n_valid)
      *(f32x4 *)((char *)(base + (size_t)(row0 + r) * H + 32 * fb) + (lane % S::LPR) * 16) = v;
  }
  wave_lds_fence();
}

// Same staging, but row r of the tile goes to row dsel (this lane's value for its own row l % 32;
// negative = the row is not stored): the rows of a tile scattered to per-row destinations.
template <typename TO, int H>
__device__ __forceinline__ void store_block_rows_via_lds(TO *base, int dsel, int fb, int lane, const f32x16 &d,
                                                         char *stage) {
  using S = BlockStage<TO>;
  const int l32 = lane & 31, g = lane >> 5;
  char *wp = stage + l32 * S::RS + 4 * g * (int)sizeof(TO);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    float v[4] = {d[4 * q], d[4 * q + 1], d[4 * q + 2], d[4 * q + 3]};
    store4<TO>((TO *)(wp + 8 * q * (int)sizeof(TO)), v);
  }
  wave_lds_fence();
#pragma unroll
  for (int k = 0; k < 32 / S::RPI; ++k) {
    const int r = k * S::RPI + lane / S::LPR;
    const int dr = __shfl(dsel, r);
    const f32x4 v = *(const f32x4 *)(stage + r * S::RS + (lane % S::LPR) * 16);
    if (dr >= 0) *(f32x4 *)((char *)(base + (size_t)dr * H + 32 * fb) + (lane % S::LPR) * 16) = v;
  }
  wave_lds_fence();
}
