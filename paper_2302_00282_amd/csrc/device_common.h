// Device-side vocabulary shared by the gfx950 kernel sources: vector types, the element-type traits (fp32 / bf16
// storage, fp32 arithmetic), bf16 conversion, and the tile constants of the MFMA GEMM loops.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include "kernels.h"

namespace xenos {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

struct bf16_t { uint16_t v; };

__device__ __forceinline__ float bf2f(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
// fp32 -> bf16, round-to-nearest-even: gfx950 converts in hardware (one packed instruction per two values)
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
__device__ __forceinline__ uint16_t f2bf(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
__device__ __forceinline__ uint32_t f2bf2(float lo, float hi) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2_t){lo, hi}, bf16x2_t));
}

template <typename T> struct Tr;
template <> struct Tr<float> {
  static constexpr int CE = 4;     // elements per 16-byte chunk
  static constexpr int BKE = kRowBytes / 4;   // reduction elements per step
  __device__ static __forceinline__ float ld(const void* p, long long i) { return ((const float*)p)[i]; }
  __device__ static __forceinline__ void st(void* p, long long i, float v) { ((float*)p)[i] = v; }
  __device__ static __forceinline__ void unpack(const u32x4_t& v, float* f) {
#pragma unroll
    for (int e = 0; e < 4; ++e) f[e] = __uint_as_float(v[e]);
  }
  __device__ static __forceinline__ u32x4_t pack(const float* f) {
    u32x4_t v;
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = __float_as_uint(f[e]);
    return v;
  }
};
template <> struct Tr<bf16_t> {
  static constexpr int CE = 8;
  static constexpr int BKE = kRowBytes / 2;
  __device__ static __forceinline__ float ld(const void* p, long long i) { return bf2f(((const uint16_t*)p)[i]); }
  __device__ static __forceinline__ void st(void* p, long long i, float v) { ((uint16_t*)p)[i] = f2bf(v); }
  __device__ static __forceinline__ void unpack(const u32x4_t& v, float* f) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      f[2 * e] = __uint_as_float(v[e] << 16);
      f[2 * e + 1] = __uint_as_float(v[e] & 0xffff0000u);
    }
  }
  __device__ static __forceinline__ u32x4_t pack(const float* f) {
    u32x4_t v;
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = f2bf2(f[2 * e], f[2 * e + 1]);
    return v;
  }
};

// max(a, b).  `fmaxf` must quiet signalling NaNs, which costs an extra `v_max x, x, x` per operand whose origin the compiler
// cannot see: values moved between lanes by DPP or unpacked from bf16 with bit operations, i.e. every operand of the
// pooling reductions (two thirds of their instructions).  fmx_raw is the bare instruction for those places; NaN inputs are
// outside the contract of the library.
__device__ __forceinline__ float fmx(float a, float b) { return __builtin_fmaxf(a, b); }
__device__ __forceinline__ float fmx_raw(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

// Two-group channel shuffle done by a store: CE finished channels of a pixel (`mine`) and the same channels of the other
// part of the concat (`oth`) alternate in the output, `first` = mine at the even positions.  Two 16-byte stores.
template <typename T>
__device__ __forceinline__ void ileave_store(T* dst, const u32x4_t& mine, const u32x4_t& oth, bool first) {
  u32x4_t w[2];
  if (sizeof(T) == 2) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t m = (mine[e >> 1] >> ((e & 1) * 16)) & 0xffffu, o = (oth[e >> 1] >> ((e & 1) * 16)) & 0xffffu;
      w[e >> 2][e & 3] = first ? (m | (o << 16)) : (o | (m << 16));
    }
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      w[e >> 1][(e & 1) * 2] = first ? mine[e] : oth[e];
      w[e >> 1][(e & 1) * 2 + 1] = first ? oth[e] : mine[e];
    }
  }
  *(u32x4_t*)dst = w[0];
  *(u32x4_t*)(dst + Tr<T>::CE) = w[1];
}

constexpr int NT = 256;          // threads per workgroup (4 wavefronts of 64)
constexpr int ROWB = kRowBytes;  // data bytes per tile row per reduction step
constexpr int CPR = ROWB / 16;   // 16-byte chunks per tile row
constexpr int KG = ROWB / 32;    // k-groups (one MFMA fragment pair each) per step
constexpr int LDS_ROW = ROWB + 16;   // row pitch in LDS: an odd number of 16-byte slots, so consecutive rows hit distinct slots
constexpr int NUM_XCD = 8;

__host__ __device__ constexpr int cmax(int a, int b) { return a > b ? a : b; }

}  // namespace xenos
