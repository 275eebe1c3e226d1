// Block form of the VLA recurrence on FP32 MFMA for the small head sizes (d = 32, 64): several heads per
// workgroup, so that the two C x C sections of a block -- dependent chains of vector instructions whose cost
// does not shrink with d -- are paid once per workgroup instead of once per head.
//
// The algebra is that of vla_chunk.hip (paper Section 3.3: eq. (sm), eq. (s-update), numerator of
// eq. (output), 16 tokens per block):
//
//   Y^T = K^ A0,  G = Y^T K^^T,  GQ = Y^T Q^T,  I + G = L L^T,  W^T = L^{-1} Y^T,  A1 = A0 - W W^T,
//   c_t = (1/L_tt) / max(||w_t|| / L_tt, eps),  F^T = V - K^ S0^T,  E^T = Z F^T with
//   Z = (I + strict_lower(L) diag(c))^{-1},  O^T = Q S0^T + NQ^T E^T with NQ[s][t] = c_s (L^{-1} GQ)[s][t]
//   for s <= t,  S1^T = S0^T + W diag(c) E^T.
//
// Work split: four waves per workgroup, 128 / d heads per workgroup (4 at d = 32, 2 at d = 64); a wave owns
// 32 columns of one head's A and the same rows of its S as accumulator tiles resident in VGPRs.  Both C x C
// sections put one head on each 16-lane row of a single wave: row r holds, lane by lane, the rows of that
// head's I + G (then of L) and the columns of L^{-1}, and every broadcast the factorisation and the two forward
// substitutions need stays inside the row (DPP row broadcast folded into the multiply-add), so one instruction
// stream serves all the heads of the workgroup.
//
// v_mfma_f32_16x16x4_f32 register layout, lane l = 16*g + c:
//   A operand: A[m = c][k = g]      B operand: B[k = g][n = c]      C/D: reg r -> D[m = 4g + r][n = c]
#include "vla_mfma_util.h"

namespace vla {
namespace {

// x[lane L of this 16-lane row]
template <int L>
__device__ __forceinline__ float row_bcast(float x) {
  float r;
  asm volatile("v_mov_b32_dpp %0, %1 row_newbcast:%2 row_mask:0xf bank_mask:0xf bound_ctrl:1"
               : "=v"(r)
               : "v"(x), "n"(L));
  return r;
}

// Cholesky of the symmetric positive definite matrix whose row c sits in lane c of every 16-lane row
// (m[s] = M[c][s]) together with X = L^{-1} by forward substitution, columns on lanes.  On exit m[s] = L[c][s]
// for s <= c (entries above the diagonal are not meaningful) and X[t] = L^{-1}[t][c].
//   step t:  L[c][t] = M[c][t] / sqrt(pivot);  M[c][j] -= L[j][t] L[c][t] for j > t   (independent updates)
//            X[t][c] = (delta_tc - sum_{s<t} L[t][s] X[s][c]) / L[t][t]               (one dependent chain)
// L[j][t] and L[t][s] are another lane's registers of the same row: DPP row broadcasts folded into the
// multiply-adds.  The two instruction streams of a step are interleaved so that the independent updates cover
// the latency of the dependent chain.
template <int T_, int I_>
__device__ __forceinline__ void chol_linv_ops(float (&m)[C], float nli, float li, const float (&nl)[C],
                                              const float (&X)[C], float& acc) {
  if constexpr (I_ < C - 1) {
    if constexpr (T_ + 1 + I_ < C) fmac_row_bcast<T_ + 1 + I_>(m[T_ + 1 + I_], nli, li);
    if constexpr (I_ < T_) fmac_row_bcast<T_>(acc, nl[I_], X[I_]);
    chol_linv_ops<T_, I_ + 1>(m, nli, li, nl, X, acc);
  }
}
template <int T_>
__device__ __forceinline__ void chol_linv_rows(float (&m)[C], float (&nl)[C], float (&X)[C], int c) {
  if constexpr (T_ < C) {
    asm volatile("s_nop 1" : "+v"(m[T_]));         // a DPP read of a VGPR needs 2 wait states after its write
    const float p = row_bcast<T_>(m[T_]);          // pivot = delta_t >= 1
    const float ri = __builtin_amdgcn_rsqf(p);     // 1 ulp; L only has to satisfy L L^T = I + G to rounding
    const float li = m[T_] * ri;                   // lane c: L[c][t]
    m[T_] = li;
    float nli = -li;
    asm volatile("s_nop 1" : "+v"(nli));
    nl[T_] = nli;
    float acc = (c == T_) ? 1.0f : 0.0f;
    chol_linv_ops<T_, 0>(m, nli, li, nl, X, acc);
    X[T_] = acc * ri;
    chol_linv_rows<T_ + 1>(m, nl, X, c);
  }
}

template <int D, typename IO, bool FMAP>
__global__ void __launch_bounds__(256, 2) chunk_multihead_kernel(ForwardArgs a) {
  constexpr int HPW = 128 / D;     // heads per workgroup
  constexpr int NWH = 4 / HPW;     // waves per head
  constexpr int SL = D / NWH;      // columns of A (rows of S) owned by one wave: 32
  constexpr int NJ = SL / 16;
  constexpr int NB = D / 16;
  constexpr int LD = D + 4;
  constexpr int NTH = 64 * NWH;    // threads per head
  constexpr int EPT = C * D / NTH; // staged elements per thread per tensor: 8
  constexpr int TPR = D / EPT;     // threads per token row
  static_assert(HPW * NWH == 4 && NJ == 2 && EPT == 8 && (TPR == 4 || TPR == 8), "layout");

  __shared__ __align__(16) float Ksb[HPW][C * LD];         // K^ [t][j]: read only before the Gram barrier
  __shared__ __align__(16) float Qsb[HPW][2][C * LD];      // Q  [t][j], double-buffered over blocks
  __shared__ __align__(16) float Ys[HPW][C * LD];          // Y^T [t][j] (each wave touches only its columns)
  __shared__ __align__(16) float Wb[HPW][D * LT];          // W   [j][t]
  __shared__ __align__(16) float Gp[HPW][NWH][2][C * LT];  // per-wave partial Gram matrices G, GQ [s][t]
  __shared__ __align__(16) float Lis[HPW][C * LT];         // L^{-1} [t][s]
  __shared__ __align__(16) float Lrs[HPW][C * LT];         // L [t][s]
  __shared__ __align__(16) float Zs[HPW][C * LT];          // Z [t][s]
  __shared__ __align__(16) float NQs[HPW][C * LT];         // -NQ^T [t][s]
  __shared__ __align__(16) float wn2p[HPW][NWH][C];        // per-wave partial ||w_t||^2
  __shared__ __align__(16) float cvec[HPW][C];             // -c_t

  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hh = w / NWH;          // head of this wave inside the workgroup
  const int wl = w % NWH;          // wave inside the head
  const int lane = tid & 63;
  const int c = lane & 15;
  const int g = lane >> 4;
  const int T = a.T;
  const float eps = a.eps;
  const int col0 = SL * wl;
  // The last workgroup may hold fewer heads than HPW: the spare waves recompute the last head (so that every
  // wave reaches every barrier with valid addresses) and store nothing.
  const int head_raw = blockIdx.x * HPW + hh;
  const bool active = head_raw < a.n_heads;
  const int head = active ? head_raw : a.n_heads - 1;

  // ---- resident state: At[b][jn][r] = A[16b + 4g + r][col0 + 16jn + c],  St likewise for S^T
  f4 At[NB][NJ], St[NB][NJ];
  {
    const float* A0 = a.A0 ? a.A0 + static_cast<size_t>(head) * D * D : nullptr;
    const float* S0 = a.S0 ? a.S0 + static_cast<size_t>(head) * D * D : nullptr;
    const float diag = 1.0f / a.lambda0;
    const int arc = (4 * g) * D + col0 + c;
    const int src = (col0 + c) * D + 4 * g;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int jn = 0; jn < NJ; ++jn) {
        if (A0) {
#pragma unroll
          for (int r = 0; r < 4; ++r) At[b][jn][r] = A0[arc + (16 * b + r) * D + 16 * jn];
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            At[b][jn][r] = (16 * b + 4 * g + r == col0 + 16 * jn + c) ? diag : 0.0f;
        }
        if (S0) {
          const float4 x = *reinterpret_cast<const float4*>(S0 + src + 16 * jn * D + 16 * b);
          St[b][jn] = f4{x.x, x.y, x.z, x.w};
        } else {
          St[b][jn] = f4{0, 0, 0, 0};
        }
      }
  }

  const size_t slab = static_cast<size_t>(head) * static_cast<size_t>(T) * D;
  const IO* qh = static_cast<const IO*>(a.q) + slab;
  const IO* kh = static_cast<const IO*>(a.k) + slab;
  const IO* vh = static_cast<const IO*>(a.v) + slab;
  IO* oh = static_cast<IO*>(a.o) + slab;

  // staging role of this thread inside its head: token row and column segment
  const int th = tid - hh * NTH;
  const int srow = th / TPR;
  const int sseg = (th % TPR) * EPT;
  const int vcol = col0 + c;

  RawRow<IO, EPT> kpre, qpre;
  IO vpre[NJ][4];

  // Loads never branch or wait: rows past the end are read from the last valid row and zeroed when consumed.
  auto load_kq = [&](int t0) {
    const int tr = t0 + srow;
    const unsigned koff = static_cast<unsigned>((tr < T ? tr : T - 1) * D + sseg);
    kpre.load(kh + koff);
    qpre.load(qh + koff);
  };
  auto load_v = [&](int t0) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int t = t0 + 4 * g + r;
      const unsigned voff = static_cast<unsigned>((t < T ? t : T - 1) * D + vcol);
#pragma unroll
      for (int jn = 0; jn < NJ; ++jn) vpre[jn][r] = vh[voff + 16 * jn];
    }
  };
  auto stage = [&](int t0, int buf) {
    float kx[EPT];
    const bool live = t0 + srow < T;
    kpre.unpack(kx);
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      if constexpr (FMAP) kx[e] = elu_plus_one(kx[e]);
      kx[e] = live ? kx[e] : 0.0f;
    }
    float ss = 0.0f;
#pragma unroll
    for (int e = 0; e < EPT; ++e) ss = fmaf(kx[e], kx[e], ss);
#pragma unroll
    for (int off = TPR / 2; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
    const float sm = fmaxf(ss, eps * eps);   // 1 / max(||k||, eps) = rsqrt(max(||k||^2, eps^2)), one Newton step
    float rn = __builtin_amdgcn_rsqf(sm);
    rn = rn * fmaf(-0.5f * sm * rn, rn, 1.5f);
#pragma unroll
    for (int e = 0; e < EPT; e += 4) {
      *reinterpret_cast<f4*>(&Ksb[hh][srow * LD + sseg + e]) =
          f4{kx[e] * rn, kx[e + 1] * rn, kx[e + 2] * rn, kx[e + 3] * rn};
    }
    qpre.unpack(kx);
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      if constexpr (FMAP) kx[e] = elu_plus_one(kx[e]);
      kx[e] = live ? kx[e] : 0.0f;
    }
#pragma unroll
    for (int e = 0; e < EPT; e += 4) {
      *reinterpret_cast<f4*>(&Qsb[hh][buf][srow * LD + sseg + e]) = f4{kx[e], kx[e + 1], kx[e + 2], kx[e + 3]};
    }
  };

  if (T > 0) {
    load_kq(0);
    load_v(0);
    stage(0, 0);
    if (C < T) load_kq(C);
  }
  __syncthreads();  // block 0 staged

  __builtin_amdgcn_s_setprio(1);
  int blk = 0;
  for (int t0 = 0; t0 < T; t0 += C, ++blk) {
    const float* Ks = Ksb[hh];
    const float* Qs = Qsb[hh][blk & 1];
    auto stage_next = [&]() {
      if (t0 + C < T) {
        stage(t0 + C, (blk + 1) & 1);
        if (t0 + 2 * C < T) load_kq(t0 + 2 * C);
      }
    };
    int cc = c;  // opaque copy: keeps lane-dependent masks from being hoisted out of the loop
    asm volatile("" : "+v"(cc));

    f4 ft[NJ];  // starts as -V^T, becomes -F^T = K^ S0^T - V^T
#pragma unroll
    for (int jn = 0; jn < NJ; ++jn)
#pragma unroll
      for (int r = 0; r < 4; ++r) ft[jn][r] = (t0 + 4 * g + r < T) ? neg_widen(vpre[jn][r]) : 0.0f;
    if (t0 + C < T) load_v(t0 + C);

    // ================= Y^T = K^ A0 -> LDS;  -F^T = K^ S0^T - V^T;  partial Gram matrices over own columns
    f4 yt[NJ];
#pragma unroll
    for (int jn = 0; jn < NJ; ++jn) yt[jn] = f4{0, 0, 0, 0};
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const f4 ka = lds4(&Ks[c * LD + 16 * b + 4 * g]);
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int jn = 0; jn < NJ; ++jn) {
          yt[jn] = mfma16(ka[r], At[b][jn][r], yt[jn]);
          ft[jn] = mfma16(ka[r], St[b][jn][r], ft[jn]);
        }
    }
#pragma unroll
    for (int jn = 0; jn < NJ; ++jn)
#pragma unroll
      for (int r = 0; r < 4; ++r) Ys[hh][(4 * g + r) * LD + col0 + 16 * jn + c] = yt[jn][r];
    {
      f4 gg[NJ], gq[NJ];
#pragma unroll
      for (int jn = 0; jn < NJ; ++jn) {
        const int o4 = c * LD + col0 + 16 * jn + 4 * g;
        const f4 ya = lds4(&Ys[hh][o4]);  // same-wave write -> read: LDS operations of one wave are ordered
        const f4 kb = lds4(&Ks[o4]);
        const f4 qb = lds4(&Qs[o4]);
        gg[jn] = f4{0, 0, 0, 0};
        gq[jn] = f4{0, 0, 0, 0};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          gg[jn] = mfma16(ya[r], kb[r], gg[jn]);
          gq[jn] = mfma16(ya[r], qb[r], gq[jn]);
        }
      }
      gg[0] += gg[1];
      gq[0] += gq[1];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        Gp[hh][wl][0][(4 * g + r) * LT + c] = gg[0][r];
        Gp[hh][wl][1][(4 * g + r) * LT + c] = gq[0][r];
      }
    }
    __syncthreads();  // (2) partial Grams visible; K^ of this block no longer needed

    // ================= C x C section 1 (one wave, one head per 16-lane row): Cholesky of I + G and L^{-1}
    const int sw = (blk + blockIdx.x) & 3;
    const int sw2 = (sw + 2) & 3;
    const int hrow = g % HPW;  // the head this lane's row serves in the C x C sections
    f4 ot[NJ];  // R^T = Q S0^T, later O^T
    auto r_pass = [&]() {
#pragma unroll
      for (int jn = 0; jn < NJ; ++jn) ot[jn] = f4{0, 0, 0, 0};
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const f4 qa = lds4(&Qs[c * LD + 16 * b + 4 * g]);
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
          for (int jn = 0; jn < NJ; ++jn) ot[jn] = mfma16(qa[r], St[b][jn][r], ot[jn]);
      }
    };
    if (w != sw) {
      __builtin_amdgcn_s_setprio(0);   // filler while wave sw factorises
      r_pass();
      stage_next();
      __builtin_amdgcn_s_setprio(1);
    } else {
      __builtin_amdgcn_s_setprio(3);   // the dependent chain is what the other waves wait for: issue it first
      float m[C];
#pragma unroll
      for (int s4 = 0; s4 < C; s4 += 4) {
        f4 acc = lds4(&Gp[hrow][0][0][c * LT + s4]);
#pragma unroll
        for (int ww = 1; ww < NWH; ++ww) acc += lds4(&Gp[hrow][ww][0][c * LT + s4]);
#pragma unroll
        for (int e = 0; e < 4; ++e) m[s4 + e] = acc[e] + ((s4 + e) == cc ? 1.0f : 0.0f);
      }
      float nl[C], X[C];
      chol_linv_rows<0>(m, nl, X, cc);
      if (g < HPW) {
#pragma unroll
        for (int t = 0; t < C; ++t) Lis[hrow][t * LT + c] = X[t];
#pragma unroll
        for (int s4 = 0; s4 < C; s4 += 4)
          *reinterpret_cast<f4*>(&Lrs[hrow][c * LT + s4]) = f4{m[s4], m[s4 + 1], m[s4 + 2], m[s4 + 3]};
      }
      __builtin_amdgcn_s_setprio(1);
    }
    __syncthreads();  // (3) L^{-1}, L visible

    // ================= W^T = L^{-1} Y^T, partial ||w_t||^2, W to LDS
    __builtin_amdgcn_s_setprio(2);   // short, and every wave of the workgroup waits on it
    const f4 la = lds4(&Lis[hh][c * LT + 4 * g]);
    f4 nwt[NJ];  // -W^T
    {
      f4 n2 = f4{0, 0, 0, 0};
#pragma unroll
      for (int jn = 0; jn < NJ; ++jn) {
        f4 acc = f4{0, 0, 0, 0};
#pragma unroll
        for (int r = 0; r < 4; ++r) acc = mfma16(la[r], yt[jn][r], acc);
        nwt[jn] = -acc;
        n2 += acc * acc;
        *reinterpret_cast<f4*>(&Wb[hh][(col0 + 16 * jn + c) * LT + 4 * g]) = acc;
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) n2[r] = row_sum16(n2[r]);
      if (c == 0) *reinterpret_cast<f4*>(&wn2p[hh][wl][4 * g]) = n2;
    }
    __builtin_amdgcn_s_setprio(1);
    __syncthreads();  // (4) W and the norm partials visible

    // ================= C x C section 2 (wave sw2, one head per 16-lane row): c_t, Z; then NQ head by head
    auto update_A = [&]() {
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const f4 wa = lds4(&Wb[hh][(16 * b + c) * LT + 4 * g]);
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
          for (int jn = 0; jn < NJ; ++jn) At[b][jn] = mfma16(wa[r], nwt[jn][r], At[b][jn]);
      }
    };
    if (w != sw2) {
      __builtin_amdgcn_s_setprio(0);
      update_A();
      __builtin_amdgcn_s_setprio(1);
    }
    if (w == sw) stage_next();
    if (w == sw2) {
      __builtin_amdgcn_s_setprio(3);
      float m[C];  // lane c: row c of this row's head's L
#pragma unroll
      for (int s4 = 0; s4 < C; s4 += 4) {
        const f4 lr = lds4(&Lrs[hrow][c * LT + s4]);
#pragma unroll
        for (int e = 0; e < 4; ++e) m[s4 + e] = lr[e];
      }
      const float dl = Lrs[hrow][c * LT + c];  // L_cc
      float wn2 = 0.0f;
#pragma unroll
      for (int ww = 0; ww < NWH; ++ww) wn2 += wn2p[hrow][ww][c];
      // hardware reciprocal and square root (1 ulp): c_t only scales the write direction
      const float rdl = __builtin_amdgcn_rcpf(dl);
      const float an = __builtin_amdgcn_sqrtf(wn2) * rdl;                // ||A_t k^_t|| = ||w_t|| / L_tt
      const float cs = rdl * __builtin_amdgcn_rcpf(fmaxf(an, eps));      // alpha^_t = c_t w_t
      if (g < HPW) cvec[hrow][c] = -cs;
      float nm[C], Zr[C];
      float ncs = -cs;
      asm volatile("s_nop 1" : "+v"(ncs));
      scale_cols<0>(m, nm, ncs);             // lane t: -L[t][s] c_s
      asm volatile("s_nop 1" : "+v"(nm[0]));
      z_rows<0>(nm, Zr, cc);
      if (g < HPW) {
#pragma unroll
        for (int t = 0; t < C; ++t) Zs[hrow][t * LT + c] = Zr[t];
      }
      // H = L^{-1} GQ (one MFMA tile per head), NQ[s][t] = c_s H[s][t] for s <= t
#pragma unroll
      for (int h2 = 0; h2 < HPW; ++h2) {
        const f4 lh = lds4(&Lis[h2][c * LT + 4 * g]);
        f4 hq = f4{0, 0, 0, 0};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          float gqv = 0.0f;
#pragma unroll
          for (int ww = 0; ww < NWH; ++ww) gqv += Gp[h2][ww][1][(4 * g + r) * LT + c];
          hq = mfma16(lh[r], gqv, hq);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int s = 4 * g + r;
          const float csr = __shfl(cs, 16 * h2 + s);   // row h2 of this wave serves head h2
          NQs[h2][c * LT + s] = (s <= c) ? -(csr * hq[r]) : 0.0f;
        }
      }
      __builtin_amdgcn_s_setprio(1);
    }
    __syncthreads();  // (5) Z, NQ, c visible

    // ================= -E^T = Z (-F^T), O^T = R^T + (-NQ^T)(-E^T), store o;  ce = diag(c) E^T
    f4 ce[NJ];
    {
      const f4 za = lds4(&Zs[hh][c * LT + 4 * g]);
#pragma unroll
      for (int jn = 0; jn < NJ; ++jn) {
        f4 et = f4{0, 0, 0, 0};
#pragma unroll
        for (int r = 0; r < 4; ++r) et = mfma16(za[r], ft[jn][r], et);
        ft[jn] = et;
      }
      if (w == sw) r_pass();
      const f4 nqa = lds4(&NQs[hh][c * LT + 4 * g]);
      const f4 cg = lds4(&cvec[hh][4 * g]);
#pragma unroll
      for (int jn = 0; jn < NJ; ++jn) {
#pragma unroll
        for (int r = 0; r < 4; ++r) ot[jn] = mfma16(nqa[r], ft[jn][r], ot[jn]);
        ce[jn] = ft[jn] * cg;
      }
      if (active) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int t = t0 + 4 * g + r;
          if (t < T) {
            const unsigned ooff = static_cast<unsigned>(t * D + vcol);
            io_store2(oh + ooff, oh + ooff + 16, ot[0][r], ot[1][r]);
          }
        }
      }
    }
    // ================= S^T += W diag(c) E^T  (and A -= W W^T on the wave that formed Z)
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const f4 wa = lds4(&Wb[hh][(16 * b + c) * LT + 4 * g]);
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int jn = 0; jn < NJ; ++jn) St[b][jn] = mfma16(wa[r], ce[jn][r], St[b][jn]);
    }
    if (w == sw2) update_A();
  }

  // ---- final state
  if (active) {
    float* AT = a.A_T ? a.A_T + static_cast<size_t>(head) * D * D : nullptr;
    float* ST = a.S_T ? a.S_T + static_cast<size_t>(head) * D * D : nullptr;
    const int arc = (4 * g) * D + col0 + c;
    const int src = (col0 + c) * D + 4 * g;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int jn = 0; jn < NJ; ++jn) {
        if (AT) {
#pragma unroll
          for (int r = 0; r < 4; ++r) AT[arc + (16 * b + r) * D + 16 * jn] = At[b][jn][r];
        }
        if (ST) {
          *reinterpret_cast<float4*>(ST + src + 16 * jn * D + 16 * b) =
              make_float4(St[b][jn][0], St[b][jn][1], St[b][jn][2], St[b][jn][3]);
        }
      }
  }
}

template <int D, typename IO>
hipError_t launch(const ForwardArgs& a, hipStream_t stream) {
  constexpr int HPW = 128 / D;
  ForwardArgs args = a;
  void* params[] = {&args};
  const void* fn = a.feature_map ? reinterpret_cast<const void*>(&chunk_multihead_kernel<D, IO, true>)
                                 : reinterpret_cast<const void*>(&chunk_multihead_kernel<D, IO, false>);
  return hipLaunchKernel(fn, dim3((a.n_heads + HPW - 1) / HPW), dim3(256), params, 0, stream);
}

}  // namespace

hipError_t launch_chunk_multihead(const ForwardArgs& a, int d, int io_dtype, hipStream_t stream) {
  const bool bf = io_dtype == 1;
  switch (d) {
    case 32: return bf ? launch<32, uint16_t>(a, stream) : launch<32, float>(a, stream);
    case 64: return bf ? launch<64, uint16_t>(a, stream) : launch<64, float>(a, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace vla
