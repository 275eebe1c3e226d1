// Token-by-token VLA scan: one workgroup per (batch, head), A and S resident in registers.
//
// Paper Section 3.3 (eq. (sm), eq. (s-update)), read-out numerator of eq. (output).
//
// Thread layout (2*D threads): thread i in [0, D) owns row i of A, thread D+i owns row i of S,
// each as D floats in VGPRs.  Tokens are staged through LDS in tiles of kTile tokens (coalesced
// global loads, bf16 widened on the way in); the per-token vectors are read back from LDS as
// broadcasts, so the matrix-vector products need no cross-lane reduction.
//
// Per token, with z' = A_{t-1} k (raw key), n = max(||k||, eps):
//   k^ = k/n, z = z'/n, delta = max(1 + (k.z')/n^2, eps),  A -= z z^T / delta
//   A_t k^ = z/delta (holds because u = k^), so alpha^ = z' * ca with
//   ca = 1 / (n delta max(||z'||/(n delta), eps))
//   e = v - (S_{t-1} k)/n,  S += e alpha^^T,  o = S_{t-1} q + e (alpha^ . q)  ( = S_t q )
// Only four scalars (k.k, k.z', z'.z', z'.q) need a cross-thread reduction, so one barrier per
// token suffices (the exchange buffers are double-buffered on token parity).
#include "vla_common.h"

namespace vla {
namespace {

constexpr int kTile = 32;  // tokens per LDS tile; even, so token parity == in-tile parity

__device__ __forceinline__ void load4(const float* p, float out[4]) {
  const float4 x = *reinterpret_cast<const float4*>(p);
  out[0] = x.x; out[1] = x.y; out[2] = x.z; out[3] = x.w;
}
__device__ __forceinline__ void load4(const uint16_t* p, float out[4]) {
  const uint2 x = *reinterpret_cast<const uint2*>(p);
  out[0] = bf16_to_f32(static_cast<uint16_t>(x.x & 0xffffu));
  out[1] = bf16_to_f32(static_cast<uint16_t>(x.x >> 16));
  out[2] = bf16_to_f32(static_cast<uint16_t>(x.y & 0xffffu));
  out[3] = bf16_to_f32(static_cast<uint16_t>(x.y >> 16));
}
__device__ __forceinline__ void store1(float* p, float x) { *p = x; }
__device__ __forceinline__ void store1(uint16_t* p, float x) { *p = f32_to_bf16_rne(x); }

// D = d_k is the length of a row of either matrix (and of q, k); DV = d_v is the number of rows of S (and the
// length of v, o).  Threads [0, D) own the rows of A, threads [D, D + DV) the rows of S.
template <int D, int DV, typename IO>
__global__ void __launch_bounds__(D + DV) scan_kernel(ForwardArgs a) {
  constexpr int NT = D + DV;
  constexpr int RED_LANES = D < 64 ? D : 64;  // A-role lanes that share one wave
  constexpr int NWA = (D + 63) / 64;          // waves publishing partial sums

  __shared__ __align__(16) float qs[kTile * D];
  __shared__ __align__(16) float ks[kTile * D];
  __shared__ __align__(16) float vs[kTile * DV];
  __shared__ __align__(16) float zb[2][D];
  __shared__ __align__(16) float red[2][NWA][4];

  const int head = blockIdx.x;
  const int tid = threadIdx.x;
  const int role = tid < D ? 0 : 1;  // 0: a row of A, 1: a row of S
  const int i = tid - role * D;
  const int T = a.T;

  float row[D];
  {
    const float* src = role == 0 ? a.A0 : a.S0;
    if (src != nullptr) {
      const float* p = src + (static_cast<size_t>(head) * (role == 0 ? D : DV) + i) * D;
#pragma unroll
      for (int j = 0; j < D; j += 4) load4(p + j, &row[j]);
    } else {
      const float diag = role == 0 ? 1.0f / a.lambda0 : 0.0f;
#pragma unroll
      for (int j = 0; j < D; ++j) row[j] = (j == i) ? diag : 0.0f;
    }
  }

  const size_t slab = static_cast<size_t>(head) * static_cast<size_t>(T) * D;
  const size_t slabv = static_cast<size_t>(head) * static_cast<size_t>(T) * DV;
  const IO* qh = static_cast<const IO*>(a.q) + slab;
  const IO* kh = static_cast<const IO*>(a.k) + slab;
  const IO* vh = static_cast<const IO*>(a.v) + slabv;
  IO* oh = static_cast<IO*>(a.o) + slabv;
  const float eps = a.eps;

  for (int t0 = 0; t0 < T; t0 += kTile) {
    const int nt = (T - t0) < kTile ? (T - t0) : kTile;
    __syncthreads();  // every thread is done with the previous tile
    for (int idx = tid; idx < nt * (D / 4); idx += NT) {
      const size_t off = static_cast<size_t>(t0) * D + static_cast<size_t>(idx) * 4;
      float x[4];
      load4(qh + off, x);
      *reinterpret_cast<float4*>(&qs[idx * 4]) = make_float4(x[0], x[1], x[2], x[3]);
      load4(kh + off, x);
      *reinterpret_cast<float4*>(&ks[idx * 4]) = make_float4(x[0], x[1], x[2], x[3]);
    }
    for (int idx = tid; idx < nt * (DV / 4); idx += NT) {
      float x[4];
      load4(vh + static_cast<size_t>(t0) * DV + static_cast<size_t>(idx) * 4, x);
      *reinterpret_cast<float4*>(&vs[idx * 4]) = make_float4(x[0], x[1], x[2], x[3]);
    }
    __syncthreads();

    for (int tt = 0; tt < nt; ++tt) {
      const int par = tt & 1;
      const float4* k4 = reinterpret_cast<const float4*>(&ks[tt * D]);
      const float4* q4 = reinterpret_cast<const float4*>(&qs[tt * D]);

      // ---- matrix-vector products against the pre-update state
      float m0 = 0.f, m1 = 0.f, m2 = 0.f, m3 = 0.f;  // role 0: z' = A k ; role 1: p' = S k
      float r0 = 0.f, r1 = 0.f, r2 = 0.f, r3 = 0.f;  // role 1: r = S q
      if (role == 0) {
#pragma unroll
        for (int j = 0; j < D; j += 4) {
          const float4 kk = k4[j / 4];
          m0 = fmaf(row[j + 0], kk.x, m0);
          m1 = fmaf(row[j + 1], kk.y, m1);
          m2 = fmaf(row[j + 2], kk.z, m2);
          m3 = fmaf(row[j + 3], kk.w, m3);
        }
      } else {
#pragma unroll
        for (int j = 0; j < D; j += 4) {
          const float4 kk = k4[j / 4];
          const float4 qq = q4[j / 4];
          m0 = fmaf(row[j + 0], kk.x, m0);
          m1 = fmaf(row[j + 1], kk.y, m1);
          m2 = fmaf(row[j + 2], kk.z, m2);
          m3 = fmaf(row[j + 3], kk.w, m3);
          r0 = fmaf(row[j + 0], qq.x, r0);
          r1 = fmaf(row[j + 1], qq.y, r1);
          r2 = fmaf(row[j + 2], qq.z, r2);
          r3 = fmaf(row[j + 3], qq.w, r3);
        }
      }
      const float mv = (m0 + m1) + (m2 + m3);
      const float rv = (r0 + r1) + (r2 + r3);

      // ---- the four scalars that need all of z': partial sums per wave, then through LDS
      float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
      if (role == 0) {
        const float ki = ks[tt * D + i];
        const float qi = qs[tt * D + i];
        s0 = ki * ki;
        s1 = ki * mv;
        s2 = mv * mv;
        s3 = mv * qi;
        zb[par][i] = mv;
      }
#pragma unroll
      for (int off = RED_LANES / 2; off >= 1; off >>= 1) {
        s0 += __shfl_xor(s0, off);
        s1 += __shfl_xor(s1, off);
        s2 += __shfl_xor(s2, off);
        s3 += __shfl_xor(s3, off);
      }
      if (role == 0 && (i % RED_LANES) == 0) {
        *reinterpret_cast<float4*>(&red[par][i / RED_LANES][0]) = make_float4(s0, s1, s2, s3);
      }
      __syncthreads();

      float kk = 0.f, kz = 0.f, zz = 0.f, zq = 0.f;
#pragma unroll
      for (int w = 0; w < NWA; ++w) {
        const float4 p = *reinterpret_cast<const float4*>(&red[par][w][0]);
        kk += p.x; kz += p.y; zz += p.z; zq += p.w;
      }
      const float n = fmaxf(sqrtf(kk), eps);
      const float inv_n = 1.0f / n;
      const float delta = fmaxf(1.0f + kz * inv_n * inv_n, eps);
      const float inv_nd = inv_n / delta;                 // z'/(n delta) = A_t k^
      const float aden = fmaxf(sqrtf(zz) * inv_nd, eps);  // max(||A_t k^||, eps)
      const float ca = inv_nd / aden;                     // alpha^ = z' * ca
      const float4* z4 = reinterpret_cast<const float4*>(&zb[par][0]);

      if (role == 0) {
        const float f = -(mv * inv_n) * inv_nd;  // -(z_i / delta)
#pragma unroll
        for (int j = 0; j < D; j += 4) {
          const float4 zj = z4[j / 4];
          row[j + 0] = fmaf(f, zj.x, row[j + 0]);
          row[j + 1] = fmaf(f, zj.y, row[j + 1]);
          row[j + 2] = fmaf(f, zj.z, row[j + 2]);
          row[j + 3] = fmaf(f, zj.w, row[j + 3]);
        }
      } else {
        const float e = vs[tt * DV + i] - mv * inv_n;
        const float g = e * ca;
#pragma unroll
        for (int j = 0; j < D; j += 4) {
          const float4 zj = z4[j / 4];
          row[j + 0] = fmaf(g, zj.x, row[j + 0]);
          row[j + 1] = fmaf(g, zj.y, row[j + 1]);
          row[j + 2] = fmaf(g, zj.z, row[j + 2]);
          row[j + 3] = fmaf(g, zj.w, row[j + 3]);
        }
        store1(oh + static_cast<size_t>(t0 + tt) * DV + i, fmaf(g, zq, rv));
      }
    }
  }

  float* dst = role == 0 ? a.A_T : a.S_T;
  if (dst != nullptr) {
    float* p = dst + (static_cast<size_t>(head) * (role == 0 ? D : DV) + i) * D;
#pragma unroll
    for (int j = 0; j < D; j += 4) {
      *reinterpret_cast<float4*>(p + j) = make_float4(row[j], row[j + 1], row[j + 2], row[j + 3]);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// General variant: all lines of Algorithm 1.  Same thread layout as scan_kernel.  Per token, with
// u~ the raw penalty direction (the key itself when none is supplied), k the key after the optional
// feature map, n_k = max(||k||, eps), n_u = max(||u~||, eps), su = u_scale / n_u:
//   z' = A u~, y' = A k               (one sweep of A_{t-1}, two accumulators)
//   delta = max(1 + su^2 (u~ . z'), eps);   A -= su^2 z' z'^T / delta;   A += eta I on refresh steps
//   a = A_t k^ = y'/n_k - z' su^2 (u~ . y') / (n_k delta)  (+ eta k^)       (A symmetric)
//   alpha^ = a / max(||a||, eps);  e = v - (S k)/n_k;  S += e alpha^^T;  o = S_{t-1} q + e (alpha^ . q)
//   zkey += k;  o /= max(q . zkey, eps)  when the read-out is normalised (eq. (output))
// Two reductions per token (a needs delta and u~ . y' first), hence two barriers per token.
constexpr int kTileG = 16;

__device__ __forceinline__ float elu1(float x) { return x > 0.0f ? x + 1.0f : expf(x); }

// D = d_k, DV = d_v as in scan_kernel: threads [0, D) own the rows of A, threads [D, D + DV) the rows of S.
template <int D, int DV, typename IO>
__global__ void __launch_bounds__(D + DV) scan_general_kernel(ForwardArgs a) {
  constexpr int NT = D + DV;
  constexpr int RED_LANES = D < 64 ? D : 64;
  constexpr int NWA = (D + 63) / 64;

  __shared__ __align__(16) float qs[kTileG * D];
  __shared__ __align__(16) float ks[kTileG * D];
  __shared__ __align__(16) float vs[kTileG * DV];
  __shared__ __align__(16) float us[kTileG * D];
  __shared__ __align__(16) float zb[2][D];   // z' (raw)
  __shared__ __align__(16) float ab[2][D];   // a = A_t k^
  __shared__ __align__(16) float red1[2][NWA][8];
  __shared__ __align__(16) float red2[2][NWA][2];

  const int head = blockIdx.x;
  const int tid = threadIdx.x;
  const int role = tid < D ? 0 : 1;
  const int i = tid - role * D;
  const int T = a.T;
  const bool has_u = a.u != nullptr;

  float row[D];
  {
    const float* src = role == 0 ? a.A0 : a.S0;
    if (src != nullptr) {
      const float* p = src + (static_cast<size_t>(head) * (role == 0 ? D : DV) + i) * D;
#pragma unroll
      for (int j = 0; j < D; j += 4) load4(p + j, &row[j]);
    } else {
      const float diag = role == 0 ? 1.0f / a.lambda0 : 0.0f;
#pragma unroll
      for (int j = 0; j < D; ++j) row[j] = (j == i) ? diag : 0.0f;
    }
  }
  float zkey = (role == 0 && a.zkey0 != nullptr) ? a.zkey0[static_cast<size_t>(head) * D + i] : 0.0f;

  const size_t slab = static_cast<size_t>(head) * static_cast<size_t>(T) * D;
  const size_t slabv = static_cast<size_t>(head) * static_cast<size_t>(T) * DV;
  const IO* qh = static_cast<const IO*>(a.q) + slab;
  const IO* kh = static_cast<const IO*>(a.k) + slab;
  const IO* vh = static_cast<const IO*>(a.v) + slabv;
  const IO* uh = has_u ? static_cast<const IO*>(a.u) + slab : kh;
  IO* oh = static_cast<IO*>(a.o) + slabv;
  const float eps = a.eps;

  for (int t0 = 0; t0 < T; t0 += kTileG) {
    const int nt = (T - t0) < kTileG ? (T - t0) : kTileG;
    __syncthreads();
    for (int idx = tid; idx < nt * (D / 4); idx += NT) {
      const size_t off = static_cast<size_t>(t0) * D + static_cast<size_t>(idx) * 4;
      float x[4];
      load4(qh + off, x);
      if (a.feature_map) { x[0] = elu1(x[0]); x[1] = elu1(x[1]); x[2] = elu1(x[2]); x[3] = elu1(x[3]); }
      *reinterpret_cast<float4*>(&qs[idx * 4]) = make_float4(x[0], x[1], x[2], x[3]);
      load4(kh + off, x);
      if (a.feature_map) { x[0] = elu1(x[0]); x[1] = elu1(x[1]); x[2] = elu1(x[2]); x[3] = elu1(x[3]); }
      *reinterpret_cast<float4*>(&ks[idx * 4]) = make_float4(x[0], x[1], x[2], x[3]);
      if (has_u) load4(uh + off, x);  // without a supplied u the penalty direction is the key as used
      *reinterpret_cast<float4*>(&us[idx * 4]) = make_float4(x[0], x[1], x[2], x[3]);
    }
    for (int idx = tid; idx < nt * (DV / 4); idx += NT) {
      float x[4];
      load4(vh + static_cast<size_t>(t0) * DV + static_cast<size_t>(idx) * 4, x);
      *reinterpret_cast<float4*>(&vs[idx * 4]) = make_float4(x[0], x[1], x[2], x[3]);
    }
    __syncthreads();

    for (int tt = 0; tt < nt; ++tt) {
      const int par = tt & 1;
      const float4* k4 = reinterpret_cast<const float4*>(&ks[tt * D]);
      const float4* q4 = reinterpret_cast<const float4*>(&qs[tt * D]);
      const float4* u4 = reinterpret_cast<const float4*>(&us[tt * D]);

      // role 0: m = z' = A u~, r = y' = A k ; role 1: m = S k, r = S q
      float m0 = 0.f, m1 = 0.f, r0 = 0.f, r1 = 0.f;
      {
        const float4* x4 = role == 0 ? u4 : k4;
        const float4* y4 = role == 0 ? k4 : q4;
#pragma unroll
        for (int j = 0; j < D; j += 4) {
          const float4 xx = x4[j / 4];
          const float4 yy = y4[j / 4];
          m0 = fmaf(row[j + 0], xx.x, m0);
          m1 = fmaf(row[j + 1], xx.y, m1);
          m0 = fmaf(row[j + 2], xx.z, m0);
          m1 = fmaf(row[j + 3], xx.w, m1);
          r0 = fmaf(row[j + 0], yy.x, r0);
          r1 = fmaf(row[j + 1], yy.y, r1);
          r0 = fmaf(row[j + 2], yy.z, r0);
          r1 = fmaf(row[j + 3], yy.w, r1);
        }
      }
      const float mv = m0 + m1;
      const float rv = r0 + r1;

      // ---- first reduction: k.k, u~.u~, u~.z', u~.y', q.zkey
      float s[5] = {0.f, 0.f, 0.f, 0.f, 0.f};
      float ki = 0.f;
      if (role == 0) {
        ki = ks[tt * D + i];
        const float ui = us[tt * D + i];
        zkey += ki;
        s[0] = ki * ki;
        s[1] = ui * ui;
        s[2] = ui * mv;
        s[3] = ui * rv;
        s[4] = qs[tt * D + i] * zkey;
        zb[par][i] = mv;
      }
#pragma unroll
      for (int off = RED_LANES / 2; off >= 1; off >>= 1) {
#pragma unroll
        for (int e = 0; e < 5; ++e) s[e] += __shfl_xor(s[e], off);
      }
      if (role == 0 && (i % RED_LANES) == 0) {
#pragma unroll
        for (int e = 0; e < 5; ++e) red1[par][i / RED_LANES][e] = s[e];
      }
      __syncthreads();

      float kk = 0.f, uu = 0.f, uz = 0.f, uy = 0.f, qz = 0.f;
#pragma unroll
      for (int w = 0; w < NWA; ++w) {
        kk += red1[par][w][0]; uu += red1[par][w][1]; uz += red1[par][w][2];
        uy += red1[par][w][3]; qz += red1[par][w][4];
      }
      const float inv_nk = 1.0f / fmaxf(sqrtf(kk), eps);
      const float su = (has_u ? a.u_scale : 1.0f) / fmaxf(sqrtf(uu), eps);  // u = k^ carries no scale
      const float su2 = su * su;
      const float delta = fmaxf(1.0f + su2 * uz, eps);
      const float cz = su2 / delta;  // A -= cz z' z'^T ;  a = y' inv_nk - z' cz (u~ . y') inv_nk
      const bool refresh = a.refresh_period > 0 && ((a.step_offset + t0 + tt + 1) % a.refresh_period) == 0;
      const float eta = refresh ? a.refresh_eta : 0.0f;
      const float4* z4 = reinterpret_cast<const float4*>(&zb[par][0]);

      // ---- second reduction: a = A_t k^ on the A threads; ||a||^2, a.q
      float t2[2] = {0.f, 0.f};
      if (role == 0) {
        const float ai = (rv - mv * cz * uy) * inv_nk + eta * ki * inv_nk;
        ab[par][i] = ai;
        t2[0] = ai * ai;
        t2[1] = ai * qs[tt * D + i];
        const float f = -mv * cz;
#pragma unroll
        for (int j = 0; j < D; j += 4) {
          const float4 zj = z4[j / 4];
          row[j + 0] = fmaf(f, zj.x, row[j + 0]);
          row[j + 1] = fmaf(f, zj.y, row[j + 1]);
          row[j + 2] = fmaf(f, zj.z, row[j + 2]);
          row[j + 3] = fmaf(f, zj.w, row[j + 3]);
        }
        if (refresh) {
#pragma unroll
          for (int j = 0; j < D; ++j) row[j] += (j == i) ? eta : 0.0f;
        }
      }
#pragma unroll
      for (int off = RED_LANES / 2; off >= 1; off >>= 1) {
        t2[0] += __shfl_xor(t2[0], off);
        t2[1] += __shfl_xor(t2[1], off);
      }
      if (role == 0 && (i % RED_LANES) == 0) {
        red2[par][i / RED_LANES][0] = t2[0];
        red2[par][i / RED_LANES][1] = t2[1];
      }
      __syncthreads();

      if (role == 1) {
        float aa = 0.f, aq = 0.f;
#pragma unroll
        for (int w = 0; w < NWA; ++w) { aa += red2[par][w][0]; aq += red2[par][w][1]; }
        const float inv_an = 1.0f / fmaxf(sqrtf(aa), eps);
        const float e = vs[tt * DV + i] - mv * inv_nk;
        const float gcoef = e * inv_an;
        const float4* a4 = reinterpret_cast<const float4*>(&ab[par][0]);
#pragma unroll
        for (int j = 0; j < D; j += 4) {
          const float4 aj = a4[j / 4];
          row[j + 0] = fmaf(gcoef, aj.x, row[j + 0]);
          row[j + 1] = fmaf(gcoef, aj.y, row[j + 1]);
          row[j + 2] = fmaf(gcoef, aj.z, row[j + 2]);
          row[j + 3] = fmaf(gcoef, aj.w, row[j + 3]);
        }
        float ov = fmaf(gcoef, aq, rv);
        if (a.normalise_output) ov /= fmaxf(qz, eps);
        store1(oh + static_cast<size_t>(t0 + tt) * DV + i, ov);
      }
    }
  }

  float* dst = role == 0 ? a.A_T : a.S_T;
  if (dst != nullptr) {
    float* p = dst + (static_cast<size_t>(head) * (role == 0 ? D : DV) + i) * D;
#pragma unroll
    for (int j = 0; j < D; j += 4) {
      *reinterpret_cast<float4*>(p + j) = make_float4(row[j], row[j + 1], row[j + 2], row[j + 3]);
    }
  }
  if (role == 0 && a.zkey_T != nullptr) a.zkey_T[static_cast<size_t>(head) * D + i] = zkey;
}

template <int D, int DV, typename IO>
hipError_t launch_general(const ForwardArgs& a, hipStream_t stream) {
  ForwardArgs args = a;
  void* params[] = {&args};
  return hipLaunchKernel(reinterpret_cast<const void*>(&scan_general_kernel<D, DV, IO>), dim3(a.n_heads),
                         dim3(D + DV), params, 0, stream);
}

template <int D, int DV, typename IO>
hipError_t launch(const ForwardArgs& a, hipStream_t stream) {
  // hipLaunchKernel reports this launch's own status; the sticky hipGetLastError() value may
  // belong to an unrelated earlier call made by the host program.
  ForwardArgs args = a;
  void* params[] = {&args};
  return hipLaunchKernel(reinterpret_cast<const void*>(&scan_kernel<D, DV, IO>), dim3(a.n_heads),
                         dim3(D + DV), params, 0, stream);
}
template <int D, int DV>
hipError_t launch_pair(const ForwardArgs& a, int io_dtype, bool general, hipStream_t stream) {
  if (general) {
    return io_dtype == 1 ? launch_general<D, DV, uint16_t>(a, stream) : launch_general<D, DV, float>(a, stream);
  }
  return io_dtype == 1 ? launch<D, DV, uint16_t>(a, stream) : launch<D, DV, float>(a, stream);
}
template <int D>
hipError_t launch_dk(const ForwardArgs& a, int d_v, int io_dtype, bool general, hipStream_t stream) {
  switch (d_v) {
    case 16: return launch_pair<D, 16>(a, io_dtype, general, stream);
    case 32: return launch_pair<D, 32>(a, io_dtype, general, stream);
    case 64: return launch_pair<D, 64>(a, io_dtype, general, stream);
    case 96: return launch_pair<D, 96>(a, io_dtype, general, stream);
    case 128: return launch_pair<D, 128>(a, io_dtype, general, stream);
    default: return hipErrorInvalidValue;
  }
}
hipError_t launch_any(const ForwardArgs& a, int d_k, int d_v, int io_dtype, bool general, hipStream_t stream) {
  switch (d_k) {
    case 16: return launch_dk<16>(a, d_v, io_dtype, general, stream);
    case 32: return launch_dk<32>(a, d_v, io_dtype, general, stream);
    case 64: return launch_dk<64>(a, d_v, io_dtype, general, stream);
    case 96: return launch_dk<96>(a, d_v, io_dtype, general, stream);
    case 128: return launch_dk<128>(a, d_v, io_dtype, general, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

// Every pair of key and value head sizes out of 16, 32, 64, 96, 128, with or without the optional lines of
// Algorithm 1.
bool scan_supported(int d_k, int d_v) {
  const auto ok = [](int d) { return d == 16 || d == 32 || d == 64 || d == 96 || d == 128; };
  return ok(d_k) && ok(d_v);
}

hipError_t launch_scan(const ForwardArgs& a, int d_k, int d_v, int io_dtype, hipStream_t stream) {
  return launch_any(a, d_k, d_v, io_dtype, false, stream);
}

hipError_t launch_scan_general(const ForwardArgs& a, int d_k, int d_v, int io_dtype, hipStream_t stream) {
  return launch_any(a, d_k, d_v, io_dtype, true, stream);
}

}  // namespace vla
