// Element types of the contractions (bf16 as raw 16-bit words, fp32) and the small device helpers
// every kernel file uses: conversions, per-type constants, 16-byte chunks, problem lookup, MFMA call.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace cdp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 v8bf16_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float v16f_t;

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
// round to nearest even, in hardware (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return __builtin_bit_cast(uint16_t, static_cast<__bf16>(f)); }

template <typename T> struct Elem;
template <> struct Elem<uint16_t> {
  static constexpr int VEC = 8;      // elements per 16-byte chunk
  static constexpr int MFMA_K = 16;  // reduction elements per MFMA
  static constexpr int KPL = 8;      // reduction elements per lane per MFMA
  __device__ static __forceinline__ float to_f32(uint16_t v) { return bf16_to_f32(v); }
  __device__ static __forceinline__ uint16_t from_f32(float f) { return f32_to_bf16(f); }
};
template <> struct Elem<float> {
  static constexpr int VEC = 4, MFMA_K = 2, KPL = 1;
  __device__ static __forceinline__ float to_f32(float v) { return v; }
  __device__ static __forceinline__ float from_f32(float f) { return f; }
};

template <typename T> __device__ __forceinline__ float ld_f32(const T* p, int64_t i) { return Elem<T>::to_f32(p[i]); }
template <typename T> __device__ __forceinline__ void st_f32(T* p, int64_t i, float v) { p[i] = Elem<T>::from_f32(v); }

template <typename T> union Chunk16 {
  uint4 v;
  uint2 h[2];
  T e[16 / sizeof(T)];
};

// Problem of a launch that owns tile number `tile` (problems are listed by ascending tile_begin).
__device__ __forceinline__ int find_problem(const GemmBatch& batch, int tile) {
  int pi = 0;
  for (int q = 1; q < batch.n; ++q)
    if (tile >= batch.p[q].tile_begin) pi = q;
  return pi;
}

// blockIdx -> logical tile so that runs of G consecutive logical tiles (neighbours in a problem's tile grid, which
// read the same operand rows) execute on one XCD and find each other's rows in its L2: consecutive workgroup ids
// are dealt round-robin to the 8 XCDs, so inside every block of 8 * G ids the k-th id that lands on XCD x takes
// logical tile x * G + k.  The ids past the last whole block keep their number.
__device__ __forceinline__ int xcd_block_cyclic(int bid, int total, int G) {
  const int block = 8 * G, whole = total - total % block;
  if (bid >= whole) return bid;
  const int s = bid / block, r = bid - s * block;
  return s * block + (r & 7) * G + (r >> 3);
}

__device__ __forceinline__ v16f_t mfma_bf16(uint4 a, uint4 b, v16f_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf16_t, a), __builtin_bit_cast(v8bf16_t, b), c, 0, 0, 0);
}

}  // namespace cdp
