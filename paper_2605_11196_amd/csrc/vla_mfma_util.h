// Small device helpers shared by the MFMA kernels (block form and two-phase) of libvla.
#pragma once

#include "vla_common.h"

namespace vla {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int C = 16;       // tokens per block
constexpr int LT = C + 4;   // row stride (floats) of the 16-column LDS arrays: conflict-free b128 rows

// Workspace of the two-phase and time-parallel modes, per head and 16-token block (floats):
//   RN  [16]       1 / max(||k_t||, eps) per token, 0 for rows past the end (k^_t = k_t * RN[t])
//   WT  [D][16]    the write directions before their scaling by c_t (w_t; alpha_t with a separate u)
//   SM  [544]      Z [16][16] | -NQ^T [16][16] | -c_t [16] | 1 / max(q_t . zkey_t, eps) [16] (normalised
//                  read-out only)
// each as one array over all blocks of the head.
constexpr int SMB = 2 * C * C + 2 * C;
__host__ __device__ constexpr size_t head_stride(int nblk, int D) {
  return static_cast<size_t>(nblk) * (C + C * D + SMB);
}
__host__ __device__ constexpr size_t off_rn(int /*nblk*/, int /*D*/) { return 0; }
__host__ __device__ constexpr size_t off_wt(int nblk, int /*D*/) { return static_cast<size_t>(nblk) * C; }
__host__ __device__ constexpr size_t off_sm(int nblk, int D) { return static_cast<size_t>(nblk) * (C + C * D); }

__device__ __forceinline__ f4 mfma16(float a, float b, f4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ float readlane(float x, int lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), lane));
}
__device__ __forceinline__ f4 lds4(const float* p) { return *reinterpret_cast<const f4*>(p); }

// Sum over the 16 lanes of a DPP row; every lane of the row gets the total.
__device__ __forceinline__ float row_sum16(float x) {
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xf, 0xf, true));   // quad_perm [1,0,3,2]
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xf, 0xf, true));   // quad_perm [2,3,0,1]
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x141, 0xf, 0xf, true));  // row_half_mirror
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x140, 0xf, 0xf, true));  // row_mirror
  return x;
}

// acc += x[lane L of this 16-lane row] * y   -- one VALU instruction (DPP row broadcast folded into the FMA)
template <int L>
__device__ __forceinline__ void fmac_row_bcast(float& acc, float x, float y) {
  asm volatile("v_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf bound_ctrl:1"
               : "+v"(acc)
               : "v"(x), "v"(y), "n"(L));
}
// x[lane L of this 16-lane row] * y
template <int L>
__device__ __forceinline__ float mul_row_bcast(float x, float y) {
  float r;
  asm volatile("v_mul_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf bound_ctrl:1"
               : "=v"(r)
               : "v"(x), "v"(y), "n"(L));
  return r;
}

// Forward substitution for Z = (I + N)^{-1}, N strictly lower triangular, columns on lanes:
// on entry nm[s] holds, in lane t of every 16-lane row, -N[t][s]; on exit Z[t] = Z[t][c] in lane c.
// Row t needs N[t][s] in every lane: that is lane t's own register, broadcast by DPP inside the FMA.
template <int T_, int S_>
struct ZRow {
  static __device__ __forceinline__ void run(const float (&nm)[C], const float (&Z)[C], float& acc) {
    if constexpr (S_ < T_) {
      fmac_row_bcast<T_>(acc, nm[S_], Z[S_]);
      ZRow<T_, S_ + 1>::run(nm, Z, acc);
    }
  }
};
template <int T_>
__device__ __forceinline__ void z_rows(const float (&nm)[C], float (&Z)[C], int c) {
  if constexpr (T_ < C) {
    float acc = (c == T_) ? 1.0f : 0.0f;
    ZRow<T_, 0>::run(nm, Z, acc);
    Z[T_] = acc;
    z_rows<T_ + 1>(nm, Z, c);
  }
}
// nm[s] = m[s] * ncs[lane s of the row]  for s = 0..C-1   (ncs = -c_s, lane-distributed)
template <int S_>
__device__ __forceinline__ void scale_cols(const float (&m)[C], float (&nm)[C], float ncs) {
  if constexpr (S_ < C) {
    nm[S_] = mul_row_bcast<S_>(ncs, m[S_]);
    scale_cols<S_ + 1>(m, nm, ncs);
  }
}

__device__ __forceinline__ void io_store(float* p, float x) { *p = x; }
__device__ __forceinline__ void io_store(uint16_t* p, float x) { *p = f32_to_bf16_rne(x); }
// Two values to two addresses.  For bf16 the pair is rounded (to nearest even) by one packed hardware
// conversion and the halves are stored separately.
__device__ __forceinline__ void io_store2(float* p0, float* p1, float x0, float x1) {
  *p0 = x0;
  *p1 = x1;
}
__device__ __forceinline__ void io_store2(uint16_t* p0, uint16_t* p1, float x0, float x1) {
  typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
  typedef float fl2 __attribute__((ext_vector_type(2)));
  const uint32_t u = __builtin_bit_cast(uint32_t, __builtin_convertvector(fl2{x0, x1}, bf2));
  *p0 = static_cast<uint16_t>(u & 0xffffu);
  *p1 = static_cast<uint16_t>(u >> 16);
}

// A staged row segment of EPT consecutive elements, held in its raw (packed) form until it is used.
template <typename IO, int EPT> struct RawRow;
template <int EPT> struct RawRow<float, EPT> {
  static_assert(EPT % 4 == 0, "whole 16-byte pieces");
  float4 v[EPT / 4];
  __device__ __forceinline__ void load(const float* p) {
#pragma unroll
    for (int e = 0; e < EPT / 4; ++e) v[e] = *reinterpret_cast<const float4*>(p + 4 * e);
  }
  // F = float, or double (every float32 value is a float64 value)
  template <typename F>
  __device__ __forceinline__ void unpack(F (&x)[EPT]) const {
#pragma unroll
    for (int e = 0; e < EPT / 4; ++e) {
      x[4 * e] = v[e].x; x[4 * e + 1] = v[e].y; x[4 * e + 2] = v[e].z; x[4 * e + 3] = v[e].w;
    }
  }
};
template <int EPT> struct RawRow<uint16_t, EPT> {
  static_assert(EPT % 4 == 0, "whole 8-byte pieces");
  static constexpr int PW = EPT % 8 == 0 ? 4 : 2;   // 32-bit words per load: 16-byte pieces, else 8-byte ones
  static constexpr int NP = EPT / (2 * PW);
  typedef uint32_t Piece __attribute__((ext_vector_type(PW)));
  Piece v[NP];
  __device__ __forceinline__ void load(const uint16_t* p) {
#pragma unroll
    for (int e = 0; e < NP; ++e) v[e] = *reinterpret_cast<const Piece*>(p + 2 * PW * e);
  }
  template <typename F>
  __device__ __forceinline__ void unpack(F (&x)[EPT]) const {
#pragma unroll
    for (int e = 0; e < NP; ++e) {
#pragma unroll
      for (int i = 0; i < PW; ++i) {
        const uint32_t u = v[e][i];
        x[2 * (PW * e + i)] = __uint_as_float(u << 16);
        x[2 * (PW * e + i) + 1] = __uint_as_float(u & 0xffff0000u);
      }
    }
  }
};
// ELU(x) + 1, the feature map of Section 3.3
__device__ __forceinline__ float elu_plus_one(float x) { return x > 0.0f ? x + 1.0f : __expf(x); }

__device__ __forceinline__ float widen(float x) { return x; }
__device__ __forceinline__ float widen(uint16_t x) { return bf16_to_f32(x); }
// -x widened to float32: for bf16 the shift and the sign flip are one shift-and-add (adding the top bit is
// flipping it).
__device__ __forceinline__ float neg_widen(float x) { return -x; }
__device__ __forceinline__ float neg_widen(uint16_t x) {
  return __uint_as_float((static_cast<uint32_t>(x) << 16) + 0x80000000u);
}

}  // namespace vla
