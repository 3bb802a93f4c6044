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
