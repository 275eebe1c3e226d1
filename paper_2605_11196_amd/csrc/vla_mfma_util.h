// Small device helpers shared by the MFMA kernels (block form and two-phase) of libvla.
#pragma once

#include "vla_common.h"

namespace vla {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int C = 16;       // tokens per block
constexpr int LT = C + 4;   // row stride (floats) of the 16-column LDS arrays: conflict-free b128 rows

__device__ __forceinline__ f4 mfma16(float a, float b, f4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ float readlane(float x, int lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), lane));
}
__device__ __forceinline__ f4 lds4(const float* p) { return *reinterpret_cast<const f4*>(p); }

__device__ __forceinline__ float io_load(const float* p) { return *p; }
__device__ __forceinline__ float io_load(const uint16_t* p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void io_store(float* p, float x) { *p = x; }
__device__ __forceinline__ void io_store(uint16_t* p, float x) { *p = f32_to_bf16_rne(x); }

// A staged row segment of EPT consecutive elements, held in its raw (packed) form until it is used.
template <typename IO, int EPT> struct RawRow;
template <int EPT> struct RawRow<float, EPT> {
  float4 v[EPT / 4];
  __device__ __forceinline__ void load(const float* p) {
#pragma unroll
    for (int e = 0; e < EPT / 4; ++e) v[e] = *reinterpret_cast<const float4*>(p + 4 * e);
  }
  __device__ __forceinline__ void zero() {
#pragma unroll
    for (int e = 0; e < EPT / 4; ++e) v[e] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  __device__ __forceinline__ void unpack(float (&x)[EPT]) const {
#pragma unroll
    for (int e = 0; e < EPT / 4; ++e) {
      x[4 * e] = v[e].x; x[4 * e + 1] = v[e].y; x[4 * e + 2] = v[e].z; x[4 * e + 3] = v[e].w;
    }
  }
};
template <int EPT> struct RawRow<uint16_t, EPT> {
  uint4 v[EPT / 8];
  __device__ __forceinline__ void load(const uint16_t* p) {
#pragma unroll
    for (int e = 0; e < EPT / 8; ++e) v[e] = *reinterpret_cast<const uint4*>(p + 8 * e);
  }
  __device__ __forceinline__ void zero() {
#pragma unroll
    for (int e = 0; e < EPT / 8; ++e) v[e] = make_uint4(0u, 0u, 0u, 0u);
  }
  __device__ __forceinline__ void unpack(float (&x)[EPT]) const {
#pragma unroll
    for (int e = 0; e < EPT / 8; ++e) {
      const uint32_t u[4] = {v[e].x, v[e].y, v[e].z, v[e].w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        x[8 * e + 2 * i] = __uint_as_float(u[i] << 16);
        x[8 * e + 2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
      }
    }
  }
};
__device__ __forceinline__ float widen(float x) { return x; }
__device__ __forceinline__ float widen(uint16_t x) { return bf16_to_f32(x); }

}  // namespace vla
