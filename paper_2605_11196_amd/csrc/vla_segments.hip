// State at the boundaries of time segments, for the time-parallel mode.
//
// With u_t = k^_t the inverse penalty matrix is an explicit inverse (paper Section 3.2, eq. (sm) is the
// Sherman-Morrison form of it):  A_t = (A_0^{-1} + sum_{s<=t} k^_s k^_s^T)^{-1}.  The sum is a plain prefix sum,
// so A at the start of every segment follows from one Gram matrix per segment and one d x d inversion, all
// independent of each other; the segments then run the exact rank-1 recurrence concurrently.  The paper
// treats the A loop as sequential (Section 3.4); this goes beyond it and is only valid without the identity
// refresh and with u = k^.  Everything here is float64 so that the boundary matrices are at least as accurate
// as the float32 chain they replace (a product of two float32 numbers is exact in float64).
//
// The S recurrence is affine in S (eq. (s-update)): S_end = S_start P + Q per segment.  P and Q come from the
// map pass of the S-rows kernel; combine_kernel composes them from left to right.
#include "vla_mfma_util.h"

namespace vla {
namespace {

constexpr int kThreads = 256;

template <typename IO> __device__ __forceinline__ double widen64(IO x);
template <> __device__ __forceinline__ double widen64<float>(float x) { return static_cast<double>(x); }
template <> __device__ __forceinline__ double widen64<uint16_t>(uint16_t x) {
  return static_cast<double>(bf16_to_f32(x));
}

// ------------------------------------------------------------------------------------------ Gram
// One workgroup per (head, segment); the last segment's matrix is never needed.  Thread (ty, tx) of a 16 x 16
// grid owns G[ty + 16 a][tx + 16 b]; tokens are normalised in float64 and staged through LDS 16 at a time.
template <int D, typename IO>
__global__ void __launch_bounds__(kThreads) gram_kernel(ForwardArgs a, double* G) {
  constexpr int NA = D / 16;
  constexpr int TT = 16;          // tokens per tile
  constexpr int LDK = D + 1;      // odd stride: the 16 partial-norm threads of a token hit different banks
  constexpr int EPT = TT * D / kThreads;  // elements of the tile each thread stages
  constexpr int TPR = D / EPT;            // threads per token row
  static_assert(EPT >= 1 && TPR >= 1 && TPR <= 64 && (TPR & (TPR - 1)) == 0, "staging layout");
  __shared__ double kt[TT * LDK];

  const int head = blockIdx.x / a.n_seg;
  const int seg = blockIdx.x - head * a.n_seg;
  if (seg == a.n_seg - 1) return;
  const int tid = threadIdx.x;
  const int ty = tid >> 4, tx = tid & 15;
  const int tb = seg * a.seg_blocks * C;
  const int te = min(a.T, tb + a.seg_blocks * C);
  const IO* kh = static_cast<const IO*>(a.k) + static_cast<size_t>(head) * static_cast<size_t>(a.T) * D;
  const double eps = static_cast<double>(a.eps);
  const int srow = tid / TPR;
  const int scol = (tid % TPR) * EPT;

  double acc[NA][NA];
#pragma unroll
  for (int i = 0; i < NA; ++i)
#pragma unroll
    for (int j = 0; j < NA; ++j) acc[i][j] = 0.0;

  for (int t0 = tb; t0 < te; t0 += TT) {
    // stage: k^ = k / max(||k||, eps) in float64; rows past the end are zero
    {
      const int t = t0 + srow;
      double x[EPT];
      double ss = 0.0;
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        x[e] = t < te ? widen64<IO>(kh[static_cast<size_t>(t) * D + scol + e]) : 0.0;
        ss = fma(x[e], x[e], ss);
      }
#pragma unroll
      for (int off = TPR / 2; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
      const double rn = 1.0 / fmax(sqrt(ss), eps);
#pragma unroll
      for (int e = 0; e < EPT; ++e) kt[srow * LDK + scol + e] = x[e] * rn;
    }
    __syncthreads();
#pragma unroll 4
    for (int tt = 0; tt < TT; ++tt) {
      double ri[NA], cj[NA];
#pragma unroll
      for (int i = 0; i < NA; ++i) {
        ri[i] = kt[tt * LDK + ty + 16 * i];
        cj[i] = kt[tt * LDK + tx + 16 * i];
      }
#pragma unroll
      for (int i = 0; i < NA; ++i)
#pragma unroll
        for (int j = 0; j < NA; ++j) acc[i][j] = fma(ri[i], cj[j], acc[i][j]);
    }
    __syncthreads();
  }

  double* Gh = G + static_cast<size_t>(blockIdx.x) * D * D;
#pragma unroll
  for (int i = 0; i < NA; ++i)
#pragma unroll
    for (int j = 0; j < NA; ++j) Gh[(ty + 16 * i) * D + tx + 16 * j] = acc[i][j];
}

// ------------------------------------------------------------------------------------------ boundary
// In-place Gauss-Jordan inverse of the symmetric positive definite D x D matrix M held in LDS with row
// stride LDM (no pivoting needed for such a matrix).  All kThreads threads call it; ends with a barrier.
template <int D, int LDM>
__device__ void invert_spd(double* M, double* colp, double* rowp) {
  constexpr int RG = kThreads / D;   // rows handled concurrently
  const int j = threadIdx.x % D;
  const int rg = threadIdx.x / D;
  for (int p = 0; p < D; ++p) {
    __syncthreads();
    const double piv = 1.0 / M[p * LDM + p];
    if (threadIdx.x < D) {
      colp[threadIdx.x] = M[threadIdx.x * LDM + p];
      rowp[threadIdx.x] = M[p * LDM + threadIdx.x] * piv;
    }
    __syncthreads();
    const double rj = rowp[j];
    for (int i = rg; i < D; i += RG) {
      double val;
      if (i == p) {
        val = (j == p) ? piv : rj;
      } else if (j == p) {
        val = -colp[i] * piv;
      } else {
        val = fma(-colp[i], rj, M[i * LDM + j]);
      }
      M[i * LDM + j] = val;
    }
  }
  __syncthreads();
}

// One workgroup per (head, segment): seg_A = inverse(inverse(A0) + sum of the Gram matrices before it).
template <int D>
__global__ void __launch_bounds__(kThreads) boundary_kernel(ForwardArgs a, const double* G, float* seg_A) {
  constexpr int LDM = D + 1;
  constexpr int RG = kThreads / D;
  __shared__ double M[D * LDM];
  __shared__ double colp[D];
  __shared__ double rowp[D];

  const int head = blockIdx.x / a.n_seg;
  const int seg = blockIdx.x - head * a.n_seg;
  const int j = threadIdx.x % D;
  const int rg = threadIdx.x / D;
  const float* A0 = a.A0 ? a.A0 + static_cast<size_t>(head) * D * D : nullptr;
  float* out = seg_A + static_cast<size_t>(blockIdx.x) * D * D;
  const float diag = 1.0f / a.lambda0;   // the same float32 value the first segment starts from

  if (seg == 0) {   // the first segment starts from the caller's A0, bit for bit
    for (int i = rg; i < D; i += RG) out[i * D + j] = A0 ? A0[i * D + j] : (i == j ? diag : 0.0f);
    return;
  }
  if (A0) {
    for (int i = rg; i < D; i += RG)
      M[i * LDM + j] = 0.5 * (static_cast<double>(A0[i * D + j]) + static_cast<double>(A0[j * D + i]));
    invert_spd<D, LDM>(M, colp, rowp);
  } else {
    for (int i = rg; i < D; i += RG) M[i * LDM + j] = (i == j) ? 1.0 / static_cast<double>(diag) : 0.0;
  }
  // every thread touches only its own elements here, so no barrier is needed before the sum
  const double* Gh = G + static_cast<size_t>(head) * a.n_seg * D * D;
  for (int i = rg; i < D; i += RG) {
    double sum = M[i * LDM + j];
    for (int s = 0; s < seg; ++s) sum += Gh[static_cast<size_t>(s) * D * D + i * D + j];
    M[i * LDM + j] = sum;
  }
  invert_spd<D, LDM>(M, colp, rowp);
  for (int i = rg; i < D; i += RG) out[i * D + j] = static_cast<float>(0.5 * (M[i * LDM + j] + M[j * LDM + i]));
}

// ------------------------------------------------------------------------------------------ combine
// One wave per (head, 16-row slab of S): x <- x P_s + Q_s for s = 0 .. n_seg-2, every intermediate written
// out as the start state of segment s+1.  x is held as accumulator tiles, xt[b][r] = S[row0 + c][16b + 4g + r],
// the layout the S-rows kernel loads its start state in; the contraction index is taken in the order
// k = 16b + 4g + r so that a tile feeds straight back as the MFMA B operand.
template <int D>
__global__ void __launch_bounds__(64) combine_kernel(ForwardArgs a, float* seg_S) {
  constexpr int NB = D / 16;
  const int head = blockIdx.x / NB;
  const int row0 = (blockIdx.x - head * NB) * 16;
  const int lane = threadIdx.x;
  const int c = lane & 15;
  const int g = lane >> 4;
  const size_t hbase = static_cast<size_t>(head) * a.n_seg;
  const int ro = (row0 + c) * D + 4 * g;   // this lane's float4 inside a d x d matrix, plus 16 b

  f4 xt[NB];
  {
    const float* S0 = a.S0 ? a.S0 + static_cast<size_t>(head) * D * D : nullptr;
    float* dst = seg_S + hbase * D * D;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      xt[b] = S0 ? *reinterpret_cast<const f4*>(S0 + ro + 16 * b) : f4{0, 0, 0, 0};
      *reinterpret_cast<f4*>(dst + ro + 16 * b) = xt[b];
    }
  }
  for (int s = 0; s + 1 < a.n_seg; ++s) {
    const float* P = a.seg_PQ + (hbase + s) * 2 * D * D;
    const float* Q = P + D * D;
    f4 nx[NB];
#pragma unroll
    for (int jb = 0; jb < NB; ++jb) nx[jb] = *reinterpret_cast<const f4*>(Q + ro + 16 * jb);
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float* prow = P + (16 * b + 4 * g + r) * D + c;   // P[k][16 jb + c]
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) nx[jb] = mfma16(prow[16 * jb], xt[b][r], nx[jb]);
      }
    float* dst = seg_S + (hbase + s + 1) * D * D;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      xt[b] = nx[b];
      *reinterpret_cast<f4*>(dst + ro + 16 * b) = xt[b];
    }
  }
}

template <int D>
hipError_t launch_boundary_d(const ForwardArgs& a, const double* G, float* seg_A, hipStream_t stream) {
  ForwardArgs args = a;
  void* params[] = {&args, &G, &seg_A};
  return hipLaunchKernel(reinterpret_cast<const void*>(&boundary_kernel<D>), dim3(a.n_heads * a.n_seg),
                         dim3(kThreads), params, 0, stream);
}
template <int D, typename IO>
hipError_t launch_gram_d(const ForwardArgs& a, double* G, hipStream_t stream) {
  ForwardArgs args = a;
  void* params[] = {&args, &G};
  return hipLaunchKernel(reinterpret_cast<const void*>(&gram_kernel<D, IO>), dim3(a.n_heads * a.n_seg),
                         dim3(kThreads), params, 0, stream);
}
template <int D>
hipError_t launch_combine_d(const ForwardArgs& a, float* seg_S, hipStream_t stream) {
  ForwardArgs args = a;
  void* params[] = {&args, &seg_S};
  return hipLaunchKernel(reinterpret_cast<const void*>(&combine_kernel<D>), dim3(a.n_heads * (D / 16)),
                         dim3(64), params, 0, stream);
}

}  // namespace

hipError_t launch_gram(const ForwardArgs& a, int d, int io_dtype, double* G, hipStream_t stream) {
  const bool bf = io_dtype == 1;
  switch (d) {
    case 32: return bf ? launch_gram_d<32, uint16_t>(a, G, stream) : launch_gram_d<32, float>(a, G, stream);
    case 64: return bf ? launch_gram_d<64, uint16_t>(a, G, stream) : launch_gram_d<64, float>(a, G, stream);
    case 128: return bf ? launch_gram_d<128, uint16_t>(a, G, stream) : launch_gram_d<128, float>(a, G, stream);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_boundary(const ForwardArgs& a, int d, const double* G, float* seg_A, hipStream_t stream) {
  switch (d) {
    case 32: return launch_boundary_d<32>(a, G, seg_A, stream);
    case 64: return launch_boundary_d<64>(a, G, seg_A, stream);
    case 128: return launch_boundary_d<128>(a, G, seg_A, stream);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_combine(const ForwardArgs& a, int d, float* seg_S, hipStream_t stream) {
  switch (d) {
    case 32: return launch_combine_d<32>(a, seg_S, stream);
    case 64: return launch_combine_d<64>(a, seg_S, stream);
    case 128: return launch_combine_d<128>(a, seg_S, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace vla
