// One decode step (T = 1) of the VLA recurrence for many heads: paper Section 3.3 (eq. (sm), eq. (s-update),
// read-out numerator of eq. (output)) applied once to a resident state (Section 7.4: the fixed-size state
// S, A is the whole memory, so generation costs one such step per token).
//
// The step reads and writes 2 d^2 floats of state per head against 10 d^2 flop: it is bound by HBM, not by
// arithmetic, so the kernel is organised around coalesced traffic.  One workgroup per head; 16 consecutive
// lanes cover one row of a matrix (d/16 consecutive floats each), so a wave instruction moves four whole rows
// and a row's dot product is a 16-lane DPP reduction.  All of A and S is requested up front (the registers
// hold both matrices), z = A k^ is the only quantity that has to cross rows, through LDS and one barrier.
//
//   n = max(||k||, eps), k^ = k / n;  z = A k^;  delta = max(1 + k^.z, eps);  A -= z z^T / delta
//   A_t k^ = z / delta (u = k^), alpha^ = (z / delta) / max(||z|| / delta, eps)
//   e = v - S k^;  S += e alpha^^T;  o = S_old q + e (alpha^ . q)   ( = S_new q )
#include "vla_mfma_util.h"

namespace vla {
namespace {

template <int N> struct Vec;
template <> struct Vec<1> { using type = float; };
template <> struct Vec<2> { typedef float type __attribute__((ext_vector_type(2))); };
template <> struct Vec<4> { typedef float type __attribute__((ext_vector_type(4))); };

// EPL consecutive floats <-> registers, in the widest pieces the alignment of d/16-float segments allows
template <int EPL>
__device__ __forceinline__ void load_seg(const float* p, float (&x)[EPL]) {
  constexpr int VW = EPL % 4 == 0 ? 4 : (EPL % 2 == 0 ? 2 : 1);
  using V = typename Vec<VW>::type;
#pragma unroll
  for (int e = 0; e < EPL; e += VW) {
    const V v = *reinterpret_cast<const V*>(p + e);
    const float* f = reinterpret_cast<const float*>(&v);
#pragma unroll
    for (int i = 0; i < VW; ++i) x[e + i] = f[i];
  }
}
template <int EPL>
__device__ __forceinline__ void store_seg(float* p, const float (&x)[EPL]) {
  constexpr int VW = EPL % 4 == 0 ? 4 : (EPL % 2 == 0 ? 2 : 1);
  using V = typename Vec<VW>::type;
#pragma unroll
  for (int e = 0; e < EPL; e += VW) {
    V v;
    float* f = reinterpret_cast<float*>(&v);
#pragma unroll
    for (int i = 0; i < VW; ++i) f[i] = x[e + i];
    *reinterpret_cast<V*>(p + e) = v;
  }
}
template <int EPL>
__device__ __forceinline__ void load_io(const float* p, float (&x)[EPL]) { load_seg<EPL>(p, x); }
template <int EPL>
__device__ __forceinline__ void load_io(const uint16_t* p, float (&x)[EPL]) {
#pragma unroll
  for (int e = 0; e < EPL; ++e) x[e] = bf16_to_f32(p[e]);
}

template <int EPL>
__device__ __forceinline__ float dot_seg(const float (&x)[EPL], const float (&y)[EPL]) {
  float s = 0.0f;
#pragma unroll
  for (int e = 0; e < EPL; ++e) s = fmaf(x[e], y[e], s);
  return s;
}

struct DecodeArgs {
  const void* q;
  const void* k;
  const void* v;
  float* S;
  float* A;
  void* o;
  float eps;
  // the optional lines of Algorithm 1 (decode_general_kernel only)
  const void* u;
  float u_scale;
  int refresh;          // 1: this step adds refresh_eta to the diagonal of A
  float refresh_eta;
  int normalise_output;
  int feature_map;
  const float* zkey0;
  float* zkey_T;
};

// DV: head size of v and o (rows of S); the waves split the DV rows of S as they split the D rows of A.
template <int D, int DV, typename IO>
__global__ void __launch_bounds__(D >= 32 ? 2 * D : 64) decode_kernel(DecodeArgs a) {
  constexpr int EPL = D / 16;                 // floats per lane per row
  constexpr int ROWS_W = D >= 32 ? 32 : D;    // rows of A per wave
  constexpr int NWV = D >= 32 ? D / 32 : 1;   // waves
  constexpr int NP = ROWS_W / 4;              // passes over A: a wave instruction covers four rows
  // The DV / 4 four-row passes over S are shared out over the waves: DV / (4 NWV) consecutive ones each where that
  // divides (kEven), else pass t goes to wave t % NWV and a wave's spare slots repeat the last pass without storing.
  constexpr int TPV = DV / 4;
  constexpr bool kEven = TPV % NWV == 0;
  constexpr int NPV = kEven ? TPV / NWV : (TPV + NWV - 1) / NWV;   // pass slots per wave
  static_assert(DV % 4 == 0 && NPV >= 1, "whole passes over S");
  __shared__ float zs[D];

  const int head = blockIdx.x;
  const int w = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int c = lane & 15;
  const int g = lane >> 4;
  const int col0 = c * EPL;
  const int row0 = ROWS_W * w + g;            // row of A in pass p: row0 + 4 p
  // row of S in pass slot p of this wave, and whether the slot holds a pass of its own
  auto s_row = [&](int p) -> int {
    if constexpr (kEven) {
      return 4 * (NPV * w + p) + g;
    } else {
      const int t = w + NWV * p;
      return 4 * (t < TPV ? t : TPV - 1) + g;
    }
  };
  auto owns = [&](int p) -> bool { return kEven || w + NWV * p < TPV; };

  float* Ah = a.A + static_cast<size_t>(head) * D * D;
  float* Sh = a.S + static_cast<size_t>(head) * DV * D;
  const IO* qh = static_cast<const IO*>(a.q) + static_cast<size_t>(head) * D;
  const IO* kh = static_cast<const IO*>(a.k) + static_cast<size_t>(head) * D;
  const IO* vh = static_cast<const IO*>(a.v) + static_cast<size_t>(head) * DV;
  IO* oh = static_cast<IO*>(a.o) + static_cast<size_t>(head) * DV;

  // everything is requested before anything is used
  float Ar[NP][EPL], Sr[NPV][EPL];
#pragma unroll
  for (int p = 0; p < NP; ++p) load_seg<EPL>(Ah + (row0 + 4 * p) * D + col0, Ar[p]);
#pragma unroll
  for (int p = 0; p < NPV; ++p) load_seg<EPL>(Sh + s_row(p) * D + col0, Sr[p]);
  float kk[EPL], qq[EPL], vr[NPV];
  load_io<EPL>(kh + col0, kk);
  load_io<EPL>(qh + col0, qq);
#pragma unroll
  for (int p = 0; p < NPV; ++p) vr[p] = widen(vh[s_row(p)]);

  const float eps = a.eps;
  const float rn = 1.0f / fmaxf(sqrtf(row_sum16(dot_seg<EPL>(kk, kk))), eps);
#pragma unroll
  for (int e = 0; e < EPL; ++e) kk[e] *= rn;   // k^

  // z = A k^ : rows of this wave, then the whole vector through LDS
  float zr[NP];
#pragma unroll
  for (int p = 0; p < NP; ++p) {
    zr[p] = row_sum16(dot_seg<EPL>(Ar[p], kk));
    if (c == 0) zs[row0 + 4 * p] = zr[p];
  }
  __syncthreads();
  float zc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) zc[e] = zs[col0 + e];

  const float delta = fmaxf(1.0f + row_sum16(dot_seg<EPL>(kk, zc)), eps);
  const float rd = 1.0f / delta;
  const float an = sqrtf(row_sum16(dot_seg<EPL>(zc, zc))) * rd;   // ||A_t k^||
  const float ca = rd / fmaxf(an, eps);
  float al[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) al[e] = zc[e] * ca;               // alpha^
  const float aq = row_sum16(dot_seg<EPL>(al, qq));

#pragma unroll
  for (int p = 0; p < NP; ++p) {
    const float f = -zr[p] * rd;
#pragma unroll
    for (int e = 0; e < EPL; ++e) Ar[p][e] = fmaf(f, zc[e], Ar[p][e]);
    store_seg<EPL>(Ah + (row0 + 4 * p) * D + col0, Ar[p]);
  }
#pragma unroll
  for (int p = 0; p < NPV; ++p) {
    const float sk = row_sum16(dot_seg<EPL>(Sr[p], kk));
    const float sq = row_sum16(dot_seg<EPL>(Sr[p], qq));
    const float er = vr[p] - sk;
#pragma unroll
    for (int e = 0; e < EPL; ++e) Sr[p][e] = fmaf(er, al[e], Sr[p][e]);
    if (owns(p)) {
      store_seg<EPL>(Sh + s_row(p) * D + col0, Sr[p]);
      if (c == 0) io_store(oh + s_row(p), fmaf(er, aq, sq));
    }
  }
}

// The same step with every line of Algorithm 1 switchable.  With u~ the raw penalty direction (the key itself
// when none is supplied), k the key after the optional feature map, n_k = max(||k||, eps), n_u = max(||u~||, eps),
// su = u_scale / n_u (1 / n_k without a supplied u):
//   z' = A u~, y' = A k           (one pass over the rows of A, two dot products each)
//   delta = max(1 + su^2 (u~ . z'), eps);   A -= su^2 z' z'^T / delta;   A += eta I on a refresh step
//   a = A_t k^ = (y' - z' su^2 (u~ . y') / delta) / n_k  (+ eta k^);   alpha^ = a / max(||a||, eps)
//   e = v - (S k) / n_k;  S += e alpha^^T;  o = S_old q + e (alpha^ . q)
//   zkey += k;  o /= max(q . zkey, eps) when the read-out is normalised (eq. (output))
__device__ __forceinline__ float elu1d(float x) { return x > 0.0f ? x + 1.0f : expf(x); }

template <int D, int DV, typename IO>
__global__ void __launch_bounds__(D >= 32 ? 2 * D : 64) decode_general_kernel(DecodeArgs a) {
  constexpr int EPL = D / 16;
  constexpr int ROWS_W = D >= 32 ? 32 : D;
  constexpr int NP = ROWS_W / 4;
  // the four-row passes over S are shared out over the waves as in decode_kernel
  constexpr int NWV = D >= 32 ? D / 32 : 1;
  constexpr int TPV = DV / 4;
  constexpr bool kEven = TPV % NWV == 0;
  constexpr int NPV = kEven ? TPV / NWV : (TPV + NWV - 1) / NWV;
  static_assert(DV % 4 == 0 && NPV >= 1, "whole passes over S");
  __shared__ float zs[D];
  __shared__ float ys[D];

  const int head = blockIdx.x;
  const int w = threadIdx.x >> 6;
  const int lane = threadIdx.x & 63;
  const int c = lane & 15;
  const int g = lane >> 4;
  const int col0 = c * EPL;
  const int row0 = ROWS_W * w + g;
  auto s_row = [&](int p) -> int {
    if constexpr (kEven) {
      return 4 * (NPV * w + p) + g;
    } else {
      const int t = w + NWV * p;
      return 4 * (t < TPV ? t : TPV - 1) + g;
    }
  };
  auto owns = [&](int p) -> bool { return kEven || w + NWV * p < TPV; };

  float* Ah = a.A + static_cast<size_t>(head) * D * D;
  float* Sh = a.S + static_cast<size_t>(head) * DV * D;
  const size_t hv = static_cast<size_t>(head) * D;
  const size_t hvv = static_cast<size_t>(head) * DV;
  const IO* qh = static_cast<const IO*>(a.q) + hv;
  const IO* kh = static_cast<const IO*>(a.k) + hv;
  const IO* vh = static_cast<const IO*>(a.v) + hvv;
  IO* oh = static_cast<IO*>(a.o) + hvv;

  float Ar[NP][EPL], Sr[NPV][EPL];
#pragma unroll
  for (int p = 0; p < NP; ++p) load_seg<EPL>(Ah + (row0 + 4 * p) * D + col0, Ar[p]);
#pragma unroll
  for (int p = 0; p < NPV; ++p) load_seg<EPL>(Sh + s_row(p) * D + col0, Sr[p]);
  float kk[EPL], qq[EPL], uu[EPL], zk[EPL], vr[NPV];
  load_io<EPL>(kh + col0, kk);
  load_io<EPL>(qh + col0, qq);
  if (a.feature_map) {
#pragma unroll
    for (int e = 0; e < EPL; ++e) { kk[e] = elu1d(kk[e]); qq[e] = elu1d(qq[e]); }
  }
  if (a.u != nullptr) {
    load_io<EPL>(static_cast<const IO*>(a.u) + hv + col0, uu);
  } else {
#pragma unroll
    for (int e = 0; e < EPL; ++e) uu[e] = kk[e];
  }
#pragma unroll
  for (int e = 0; e < EPL; ++e) zk[e] = (a.zkey0 ? a.zkey0[hv + col0 + e] : 0.0f) + kk[e];   // key sum after this token
#pragma unroll
  for (int p = 0; p < NPV; ++p) vr[p] = widen(vh[s_row(p)]);

  const float eps = a.eps;
  const float inv_nk = 1.0f / fmaxf(sqrtf(row_sum16(dot_seg<EPL>(kk, kk))), eps);
  const float su = (a.u != nullptr ? a.u_scale : 1.0f) / fmaxf(sqrtf(row_sum16(dot_seg<EPL>(uu, uu))), eps);
  const float su2 = su * su;

  float zr[NP];
#pragma unroll
  for (int p = 0; p < NP; ++p) {
    zr[p] = row_sum16(dot_seg<EPL>(Ar[p], uu));
    const float yr = row_sum16(dot_seg<EPL>(Ar[p], kk));
    if (c == 0) {
      zs[row0 + 4 * p] = zr[p];
      ys[row0 + 4 * p] = yr;
    }
  }
  __syncthreads();
  float zc[EPL], yc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    zc[e] = zs[col0 + e];
    yc[e] = ys[col0 + e];
  }
  const float uz = row_sum16(dot_seg<EPL>(uu, zc));
  const float uy = row_sum16(dot_seg<EPL>(uu, yc));
  const float delta = fmaxf(1.0f + su2 * uz, eps);
  const float cz = su2 / delta;
  const float eta = a.refresh ? a.refresh_eta : 0.0f;
  float al[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) al[e] = (yc[e] - zc[e] * cz * uy) * inv_nk + eta * kk[e] * inv_nk;   // a = A_t k^
  const float inv_an = 1.0f / fmaxf(sqrtf(row_sum16(dot_seg<EPL>(al, al))), eps);
#pragma unroll
  for (int e = 0; e < EPL; ++e) al[e] *= inv_an;                                                       // alpha^
  const float aq = row_sum16(dot_seg<EPL>(al, qq));
  const float qz = row_sum16(dot_seg<EPL>(qq, zk));
  const float onorm = a.normalise_output ? 1.0f / fmaxf(qz, eps) : 1.0f;

#pragma unroll
  for (int p = 0; p < NP; ++p) {
    const float f = -zr[p] * cz;
    const int row = row0 + 4 * p;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      Ar[p][e] = fmaf(f, zc[e], Ar[p][e]);
      Ar[p][e] += (row == col0 + e) ? eta : 0.0f;
    }
    store_seg<EPL>(Ah + row * D + col0, Ar[p]);
  }
#pragma unroll
  for (int p = 0; p < NPV; ++p) {
    const float sk = row_sum16(dot_seg<EPL>(Sr[p], kk)) * inv_nk;
    const float sq = row_sum16(dot_seg<EPL>(Sr[p], qq));
    const float er = vr[p] - sk;
#pragma unroll
    for (int e = 0; e < EPL; ++e) Sr[p][e] = fmaf(er, al[e], Sr[p][e]);
    if (owns(p)) {
      store_seg<EPL>(Sh + s_row(p) * D + col0, Sr[p]);
      if (c == 0) io_store(oh + s_row(p), fmaf(er, aq, sq) * onorm);
    }
  }
  if (a.zkey_T != nullptr && w == 0 && g == 0) {
#pragma unroll
    for (int e = 0; e < EPL; ++e) a.zkey_T[hv + col0 + e] = zk[e];
  }
}

template <int D, typename IO>
hipError_t launch(const DecodeArgs& a, int n_heads, hipStream_t stream) {
  DecodeArgs args = a;
  void* params[] = {&args};
  const bool general = a.u != nullptr || a.refresh != 0 || a.normalise_output != 0 || a.feature_map != 0 ||
                       a.zkey0 != nullptr || a.zkey_T != nullptr;
  const void* fn = general ? reinterpret_cast<const void*>(&decode_general_kernel<D, D, IO>)
                           : reinterpret_cast<const void*>(&decode_kernel<D, D, IO>);
  return hipLaunchKernel(fn, dim3(n_heads), dim3(D >= 32 ? 2 * D : 64), params, 0, stream);
}
// value heads of another size than the key heads
template <int D, int DV>
hipError_t launch_rect(const DecodeArgs& a, int n_heads, int io_dtype, hipStream_t stream) {
  DecodeArgs args = a;
  void* params[] = {&args};
  const bool general = a.u != nullptr || a.refresh != 0 || a.normalise_output != 0 || a.feature_map != 0 ||
                       a.zkey0 != nullptr || a.zkey_T != nullptr;
  const void* fn =
      general ? (io_dtype == 1 ? reinterpret_cast<const void*>(&decode_general_kernel<D, DV, uint16_t>)
                               : reinterpret_cast<const void*>(&decode_general_kernel<D, DV, float>))
              : (io_dtype == 1 ? reinterpret_cast<const void*>(&decode_kernel<D, DV, uint16_t>)
                               : reinterpret_cast<const void*>(&decode_kernel<D, DV, float>));
  return hipLaunchKernel(fn, dim3(n_heads), dim3(D >= 32 ? 2 * D : 64), params, 0, stream);
}

}  // namespace

// Every pair of head sizes with or without options (the waves share out the four-row passes over S evenly where
// the counts divide, in turn where they do not).
bool decode_supported(int d_k, int d_v, bool options) {
  const auto ok = [](int d) { return d == 16 || d == 32 || d == 64 || d == 96 || d == 128; };
  if (!ok(d_k) || !ok(d_v)) return false;
  (void)options;
  return true;
}

hipError_t launch_decode(const void* q, const void* k, const void* v, float* S, float* A, void* o,
                         int n_heads, int d, int d_v, int io_dtype, const ForwardArgs& opt,
                         hipStream_t stream) {
  const bool refresh = opt.refresh_period > 0 && ((opt.step_offset + 1) % opt.refresh_period) == 0;
  const DecodeArgs a{q, k, v, S, A, o, opt.eps, opt.u, opt.u_scale, refresh ? 1 : 0, opt.refresh_eta,
                     opt.normalise_output, opt.feature_map, opt.zkey0, opt.zkey_T};
  const bool bf = io_dtype == 1;
  if (d != d_v) {
    switch (d * 1000 + d_v) {
#define VLA_RECT(DK, DVV) case DK * 1000 + DVV: return launch_rect<DK, DVV>(a, n_heads, io_dtype, stream);
      VLA_RECT(16, 32) VLA_RECT(16, 64) VLA_RECT(16, 96) VLA_RECT(16, 128)
      VLA_RECT(32, 16) VLA_RECT(32, 64) VLA_RECT(32, 96) VLA_RECT(32, 128)
      VLA_RECT(64, 16) VLA_RECT(64, 32) VLA_RECT(64, 96) VLA_RECT(64, 128)
      VLA_RECT(128, 16) VLA_RECT(128, 32) VLA_RECT(128, 64) VLA_RECT(128, 96)
      VLA_RECT(96, 16) VLA_RECT(96, 32) VLA_RECT(96, 64) VLA_RECT(96, 128)
#undef VLA_RECT
      default: return hipErrorInvalidValue;
    }
  }
  switch (d) {
    case 16: return bf ? launch<16, uint16_t>(a, n_heads, stream) : launch<16, float>(a, n_heads, stream);
    case 32: return bf ? launch<32, uint16_t>(a, n_heads, stream) : launch<32, float>(a, n_heads, stream);
    case 64: return bf ? launch<64, uint16_t>(a, n_heads, stream) : launch<64, float>(a, n_heads, stream);
    case 96: return bf ? launch<96, uint16_t>(a, n_heads, stream) : launch<96, float>(a, n_heads, stream);
    case 128: return bf ? launch<128, uint16_t>(a, n_heads, stream) : launch<128, float>(a, n_heads, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace vla
