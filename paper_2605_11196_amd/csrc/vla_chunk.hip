// Block ("chunked") form of the VLA recurrence on FP32 MFMA, 16 tokens per block.
//
// Same recurrence as paper Section 3.3 (eq. (sm), eq. (s-update)) and the read-out numerator of
// eq. (output); within a block of C = 16 tokens the token-by-token matrix-vector work is regrouped
// into dense products, which is exact algebra (results differ only in float32 rounding order).
//
// With A0, S0 the state entering the block, K^ (C x d) the normalised keys, Q, V the queries and
// values of the block (rows = tokens), and u = k^:
//
//   Y^T = K^ A0                                   (C x d)      z before the in-block corrections
//   G   = Y^T K^^T ,  GQ = Y^T Q^T                (C x C)      Gram matrices in the A0 metric
//   I + G = L L^T                                 (Cholesky)   L_tt = sqrt(delta_t), L_ts = w_s . k^_t
//   W^T = L^{-1} Y^T                              (C x d)      w_t = z_t / sqrt(delta_t)
//   A1  = A0 - W W^T                                           C Sherman-Morrison steps at once
//   alpha^_t = c_t w_t ,  c_t = (1/L_tt) / max(||w_t|| / L_tt, eps)       (A_t k^_t = w_t / L_tt)
//   F^T = V - K^ S0^T                             (C x d_v)    residuals against the entering state
//   E^T = Z F^T ,  Z = (I + strict_lower(L) diag(c))^{-1}      residuals e_t of the recurrence
//   O^T = Q S0^T + NQ^T E^T ,  NQ[s][t] = c_s (L^{-1} GQ)[s][t] for s <= t, else 0
//   S1^T = S0^T + W diag(c) E^T
//
// A zero key gives an all-zero row in Y, W and E, so padding the last block with zero tokens is exact.
//
// Work split: NW waves per (batch, head); wave w owns columns [SL*w, SL*w+SL) of A and the same rows of
// S, as 16x16 MFMA accumulator tiles that stay in VGPRs for the whole sequence (A is symmetric, so an
// accumulator tile of A can be fed straight back as the B operand).  The C x C factorisations run on
// one wave (rotating with the block index) with lanes = rows and v_readlane broadcasts.
//
// v_mfma_f32_16x16x4_f32 register layout, lane l = 16*g + c:
//   A operand: A[m = c][k = g]      B operand: B[k = g][n = c]      C/D: reg r -> D[m = 4g + r][n = c]
#include "vla_mfma_util.h"

namespace vla {
namespace {

// Wave priority: LEVELS = 2: the full scheme (level FULL); 1: only the serial chains are raised (level CHAIN at
// their start and end, nothing where CHAIN < 0); 0: every wave stays at the default priority.
template <int LEVELS, int FULL, int CHAIN>
__device__ __forceinline__ void prio() {
  if constexpr (LEVELS == 2) __builtin_amdgcn_s_setprio(FULL);
  else if constexpr (LEVELS == 1 && CHAIN >= 0) __builtin_amdgcn_s_setprio(CHAIN);
}

// FMAP: q and k are replaced by ELU(x) + 1 while they are staged (the feature map of Section 3.3).
// DV: head size of v and o (rows of S); the wave that owns columns [SL w, SL w + SL) of A owns rows
// [SLV w, SLV w + SLV) of S.
template <int D, int DV, int NW, typename IO, bool FMAP>
__global__ void __launch_bounds__(64 * NW, 2) chunk_kernel(ForwardArgs a) {
  // Measured at 2048 heads, T = 8192: the full scheme gains 5 % with four waves (d = 128), 1 % with three (d = 96),
  // 1-5 % with one (d = 16, 32); two-wave workgroups (d = 64), four of which share a compute unit, lose up to
  // 20 % with any of it (1536 heads: 7.0 -> 8.5 ms) and stay at the default priority.
  constexpr int kLevels = NW == 2 ? 0 : 2;
  constexpr int SL = D / NW;       // columns of A owned by one wave
  constexpr int NJ = SL / 16;      // 16-wide tiles in a slab of A
  // The DV / 16 row tiles of S are shared out over the waves: DV / (16 NW) consecutive tiles each where that
  // divides (kEven), else tile t goes to wave t % NW, and a wave with fewer tiles than the others (or none)
  // runs its spare slots on a copy of the last tile and stores nothing from them.
  constexpr int TV = DV / 16;
  constexpr bool kEven = TV % NW == 0;
  constexpr int NJV = kEven ? TV / NW : (TV + NW - 1) / NW;   // tile slots per wave
  static_assert(DV % 16 == 0 && NJV >= 1, "whole tiles of S");
  constexpr int NB = D / 16;       // 16-row blocks over the whole head dimension
  constexpr int LD = D + 4;        // row stride of the token-major LDS arrays
  constexpr int NT = 64 * NW;
  // Staging: a token row is split over TPR threads of EPT elements each.  For the power-of-two head sizes every
  // thread stages; at d = 96 a row takes 6 threads of 16 elements in a group of 8 (two lanes of each group and
  // the third wave stage nothing), so that a row never straddles a wave and sums with a power-of-two shuffle.
  constexpr int TPR0 = NT / C;                   // thread slots per row when every thread stages
  constexpr bool PADDED = (TPR0 & (TPR0 - 1)) != 0;
  constexpr int EPT = PADDED ? 16 : C * D / NT;  // staged elements per thread per tensor
  constexpr int TPR = PADDED ? 8 : D / EPT;      // thread slots per token row
  static_assert(EPT % 4 == 0 && TPR <= 16 && (TPR & (TPR - 1)) == 0 && C * TPR <= NT && D % EPT == 0 &&
                D / EPT <= TPR, "staging layout");

  __shared__ __align__(16) float Ksb[2][C * LD];      // K^  [t][j], double-buffered over blocks
  __shared__ __align__(16) float Qsb[2][C * LD];      // Q   [t][j]
  __shared__ __align__(16) float Ys[C * LD];          // Y^T [t][j] (each wave touches only its columns)
  __shared__ __align__(16) float Wb[D * LT];          // W   [j][t]
  __shared__ __align__(16) float Gp[NW][2][C * LT];   // per-wave partial Gram matrices G, GQ  [s][t]
  __shared__ __align__(16) float Lis[C * LT];         // L^{-1} [t][s]
  __shared__ __align__(16) float Lrs[C * LT];         // L [t][s] (rows), for the wave that forms Z
  __shared__ __align__(16) float Zs[C * LT];          // Z   [t][s]
  __shared__ __align__(16) float NQs[C * LT];         // -NQ^T [t][s]
  __shared__ __align__(16) float wn2p[NW][C];         // per-wave partial ||w_t||^2
  __shared__ __align__(16) float cvec[C];             // -c_t

  const int head = blockIdx.x;
  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave index, known to be uniform
  const int lane = tid & 63;
  const int c = lane & 15;
  const int g = lane >> 4;
  const int T = a.T;
  const float eps = a.eps;
  const int col0 = SL * w;    // first column of this wave's slab of A
  const int row0 = 16 * NJV * w;   // kEven: first row of this wave's slab of S
  // first S row of this wave's tile slot jn, and whether the slot holds a tile of its own
  auto s_row = [&](int jn) -> int {
    if constexpr (kEven) {
      return row0 + 16 * jn;
    } else {
      const int t = w + NW * jn;
      return 16 * (t < TV ? t : TV - 1);
    }
  };
  auto owns = [&](int jn) -> bool { return kEven || w + NW * jn < TV; };

  // ---- resident state: accumulator tiles
  // At[b][jn][r] = A[16b + 4g + r][col0 + 16jn + c]
  // St[b][jn][r] = S[row0 + 16jn + c][16b + 4g + r]      (i.e. tiles of S^T)
  f4 At[NB][NJ], St[NB][NJV];
  {
    const float* A0 = a.A0 ? a.A0 + static_cast<size_t>(head) * D * D : nullptr;
    const float* S0 = a.S0 ? a.S0 + static_cast<size_t>(head) * DV * D : nullptr;
    const float diag = 1.0f / a.lambda0;
    const int arc = (4 * g) * D + col0 + c;  // A[4g][col0 + c]
    const int src = c * D + 4 * g;  // S[c][4g]
#pragma unroll
    for (int b = 0; b < NB; ++b) {
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
      }
#pragma unroll
      for (int jn = 0; jn < NJV; ++jn) {
        if (S0) {
          const float4 x = *reinterpret_cast<const float4*>(S0 + src + s_row(jn) * D + 16 * b);
          St[b][jn] = f4{x.x, x.y, x.z, x.w};
        } else {
          St[b][jn] = f4{0, 0, 0, 0};
        }
      }
    }
  }

  const size_t slab = static_cast<size_t>(head) * static_cast<size_t>(T) * D;
  const size_t slab_v = static_cast<size_t>(head) * static_cast<size_t>(T) * DV;
  const IO* qh = static_cast<const IO*>(a.q) + slab;
  const IO* kh = static_cast<const IO*>(a.k) + slab;
  const IO* vh = static_cast<const IO*>(a.v) + slab_v;
  IO* oh = static_cast<IO*>(a.o) + slab_v;

  // staging role of this thread: token row and column segment
  const int srow = tid / TPR;
  const int sseg = (tid % TPR) * EPT;
  const bool stager = !PADDED || (tid < C * TPR && sseg < D);    // this thread holds a row segment
  const bool stage_wave = !PADDED || tid < C * TPR;              // uniform per wave
  const int vcol = s_row(0) + c;  // first element of a v / o row this lane touches in accumulator layout

  RawRow<IO, EPT> kpre, qpre;
  IO vpre[NJV][4];  // V^T in accumulator layout: V[t0 + 4g + r][row0 + 16jn + c]

  // Loads never branch or wait: rows past the end are read from the last valid row and replaced by
  // zeros when the registers are consumed (later).  Offsets are 32-bit from the per-head base pointers.
  auto load_kq = [&](int t0) {
    if (stager) {
      const int tr = t0 + srow;
      const unsigned koff = static_cast<unsigned>((tr < T ? tr : T - 1) * D + sseg);
      kpre.load(kh + koff);
      qpre.load(qh + koff);
    }
  };
  auto load_v = [&](int t0) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int t = t0 + 4 * g + r;
      const unsigned voff = static_cast<unsigned>((t < T ? t : T - 1) * DV + vcol);
#pragma unroll
      for (int jn = 0; jn < NJV; ++jn) vpre[jn][r] = vh[voff + (s_row(jn) - s_row(0))];
    }
  };
  // normalise this thread's share of the keys of the block starting at t0 and put K^, Q into LDS half `buf`
  auto stage = [&](int t0, int buf) {
    if (!stage_wave) return;
    float kx[EPT];
    const bool ragged = t0 + C > T;   // uniform: only the last block can hold rows past the end
    const bool live = t0 + srow < T && stager;  // rows past the end of the sequence become zero tokens
    if (stager) {
      kpre.unpack(kx);
    } else {
#pragma unroll
      for (int e = 0; e < EPT; ++e) kx[e] = 0.0f;
    }
    if constexpr (FMAP) {
#pragma unroll
      for (int e = 0; e < EPT; ++e) kx[e] = elu_plus_one(kx[e]);
    }
    if (ragged || PADDED) {
#pragma unroll
      for (int e = 0; e < EPT; ++e) kx[e] = live ? kx[e] : 0.0f;
    }
    float ss = 0.0f;
#pragma unroll
    for (int e = 0; e < EPT; ++e) ss = fmaf(kx[e], kx[e], ss);
    // the TPR = 16 threads of a token row are one DPP row; 1 / max(||k||, eps) = rsqrt(max(||k||^2, eps^2)),
    // hardware reciprocal square root refined by one Newton step
    if constexpr (TPR == 16) {
      ss = row_sum16(ss);
    } else {
#pragma unroll
      for (int off = TPR / 2; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
    }
    const float sm = fmaxf(ss, eps * eps);
    float rn = __builtin_amdgcn_rsqf(sm);
    rn = rn * fmaf(-0.5f * sm * rn, rn, 1.5f);
    if (!stager) return;
#pragma unroll
    for (int e = 0; e < EPT; e += 4) {
      *reinterpret_cast<f4*>(&Ksb[buf][srow * LD + sseg + e]) =
          f4{kx[e] * rn, kx[e + 1] * rn, kx[e + 2] * rn, kx[e + 3] * rn};
    }
    qpre.unpack(kx);
    if constexpr (FMAP) {
#pragma unroll
      for (int e = 0; e < EPT; ++e) kx[e] = elu_plus_one(kx[e]);
    }
    if (ragged) {
#pragma unroll
      for (int e = 0; e < EPT; ++e) kx[e] = live ? kx[e] : 0.0f;
    }
#pragma unroll
    for (int e = 0; e < EPT; e += 4) {
      *reinterpret_cast<f4*>(&Qsb[buf][srow * LD + sseg + e]) = f4{kx[e], kx[e + 1], kx[e + 2], kx[e + 3]};
    }
  };

  if (T > 0) {
    load_kq(0);
    load_v(0);
    stage(0, 0);
    if (C < T) load_kq(C);
  }
  __syncthreads();  // block 0 staged

  prio<kLevels, 1, -1>();
  int blk = 0;
  for (int t0 = 0; t0 < T; t0 += C, ++blk) {
    const float* Ks = Ksb[blk & 1];
    const float* Qs = Qsb[blk & 1];
    // staging of the next block (this thread's share): done where this wave is not on the critical path
    auto stage_next = [&]() {
      if (t0 + C < T) {
        stage(t0 + C, (blk + 1) & 1);
        if (t0 + 2 * C < T) load_kq(t0 + 2 * C);
      }
    };
    f4 ft[NJV];  // starts as -V^T, becomes -F^T = K^ S0^T - V^T
#pragma unroll
    for (int jn = 0; jn < NJV; ++jn)
#pragma unroll
      for (int r = 0; r < 4; ++r) ft[jn][r] = neg_widen(vpre[jn][r]);
    if (t0 + C > T) {  // uniform: rows past the end of the sequence are zero tokens
#pragma unroll
      for (int jn = 0; jn < NJV; ++jn)
#pragma unroll
        for (int r = 0; r < 4; ++r) ft[jn][r] = (t0 + 4 * g + r < T) ? ft[jn][r] : 0.0f;
    }
    if (t0 + C < T) load_v(t0 + C);

    // ================= Y^T = K^ A0 (this wave's columns); Y^T goes to LDS for the Gram products
    f4 yt[NJ];
#pragma unroll
    for (int jn = 0; jn < NJ; ++jn) yt[jn] = f4{0, 0, 0, 0};
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const f4 ka = lds4(&Ks[c * LD + 16 * b + 4 * g]);
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int jn = 0; jn < NJ; ++jn) yt[jn] = mfma16(ka[r], At[b][jn][r], yt[jn]);
    }
#pragma unroll
    for (int jn = 0; jn < NJ; ++jn)
#pragma unroll
      for (int r = 0; r < 4; ++r) Ys[(4 * g + r) * LD + col0 + 16 * jn + c] = yt[jn][r];
    // ================= -F^T = K^ S0^T - V^T  (covers the LDS round trip of Y^T)
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const f4 ka = lds4(&Ks[c * LD + 16 * b + 4 * g]);
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int jn = 0; jn < NJV; ++jn) ft[jn] = mfma16(ka[r], St[b][jn][r], ft[jn]);
    }
    // ================= partial Gram matrices over this wave's columns (independent accumulators)
    {
      f4 gg[NJ], gq[NJ];
#pragma unroll
      for (int jn = 0; jn < NJ; ++jn) {
        const int o4 = c * LD + col0 + 16 * jn + 4 * g;
        const f4 ya = lds4(&Ys[o4]);  // same-wave write -> read: LDS operations of one wave are ordered
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
#pragma unroll
      for (int jn = 1; jn < NJ; ++jn) { gg[0] += gg[jn]; gq[0] += gq[jn]; }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        Gp[w][0][(4 * g + r) * LT + c] = gg[0][r];
        Gp[w][1][(4 * g + r) * LT + c] = gq[0][r];
      }
    }
    __syncthreads();  // (2) partial Grams visible

    // ================= C x C factorisation, phase 1 (one wave): Cholesky of I + G and L^{-1}
    const int sw = (blk + head) % NW;   // wave factorising I + G this block (rotates over waves/SIMDs)
    const int sw2 = (sw + NW / 2) % NW;  // a different wave forms c, Z, NQ
    // Lanes 0-31 hold rows of I + G (-> rows of L), lanes 32-63 hold columns of the identity
    // (-> columns of L^{-1}); both halves are updated by the same instruction stream: one broadcast of
    // L[j][t] serves the Cholesky trailing update and the forward substitution for L^{-1}.
    int cc = c;  // opaque copy: keeps the (c == t) masks from being hoisted into 16 registers
    asm volatile("" : "+v"(cc));
    f4 ot[NJV];  // R^T = Q S0^T, later O^T
    auto r_pass = [&]() {
#pragma unroll
      for (int jn = 0; jn < NJV; ++jn) ot[jn] = f4{0, 0, 0, 0};
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const f4 qa = lds4(&Qs[c * LD + 16 * b + 4 * g]);
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
          for (int jn = 0; jn < NJV; ++jn) ot[jn] = mfma16(qa[r], St[b][jn][r], ot[jn]);
      }
    };
    if (w != sw) {  // the other waves use the matrix pipes while wave sw factorises
      prio<kLevels, 0, -1>();
      r_pass();
      stage_next();
      prio<kLevels, 1, -1>();
    }
    if (w == sw) {
      prio<kLevels, 3, 3>();   // the dependent chain is what the other waves wait for: issue it first
      float m[C];  // lanes <32, lane c: row c of L;  lanes >=32, lane c: m[t] = L^{-1}[t][c]
      const bool lower = lane < 32;
#pragma unroll
      for (int s4 = 0; s4 < C; s4 += 4) {
        f4 acc = lds4(&Gp[0][0][c * LT + s4]);
#pragma unroll
        for (int ww = 1; ww < NW; ++ww) acc += lds4(&Gp[ww][0][c * LT + s4]);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          m[s4 + e] = (lower ? acc[e] : 0.0f) + ((s4 + e) == cc ? 1.0f : 0.0f);
      }
#pragma unroll
      for (int t = 0; t < C; ++t) {
        const float p = readlane(m[t], t);  // pivot = delta_t >= 1
        const float ri = __builtin_amdgcn_rsqf(p);  // 1 ulp; L only has to satisfy L L^T = I + G to rounding
        const float li = m[t] * ri;  // lanes <32: column t of L;  lanes >=32: row t of L^{-1}, final
        m[t] = li;
#pragma unroll
        for (int j = t + 1; j < C; ++j) m[j] = fmaf(-li, readlane(li, j), m[j]);
      }
      if (g == 2) {
#pragma unroll
        for (int t = 0; t < C; ++t) Lis[t * LT + c] = m[t];
      }
      if (g == 0) {
#pragma unroll
        for (int s4 = 0; s4 < C; s4 += 4)
          *reinterpret_cast<f4*>(&Lrs[c * LT + s4]) = f4{m[s4], m[s4 + 1], m[s4 + 2], m[s4 + 3]};
      }
      prio<kLevels, 1, 0>();
    }
    __syncthreads();  // (3) L^{-1} visible

    // ================= W^T = L^{-1} Y^T, partial ||w_t||^2, W to LDS
    prio<kLevels, 2, -1>();
    const f4 la = lds4(&Lis[c * LT + 4 * g]);
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
        *reinterpret_cast<f4*>(&Wb[(col0 + 16 * jn + c) * LT + 4 * g]) = acc;
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) n2[r] = row_sum16(n2[r]);
      if (c == 0) *reinterpret_cast<f4*>(&wn2p[w][4 * g]) = n2;
    }
    prio<kLevels, 1, -1>();
    __syncthreads();  // (4) W and the norm partials visible

    // ================= phase 2 (wave sw2): c_t, Z, NQ -- the other waves update A meanwhile
    auto update_A = [&]() {
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const f4 wa = lds4(&Wb[(16 * b + c) * LT + 4 * g]);
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
          for (int jn = 0; jn < NJ; ++jn) At[b][jn] = mfma16(wa[r], nwt[jn][r], At[b][jn]);
      }
    };
    if (w != sw2) {
      prio<kLevels, 0, -1>();
      update_A();
      prio<kLevels, 1, -1>();
    }
    if (w == sw) stage_next();  // (sw != sw2 when NW > 1)
    if (w == sw2) {
      prio<kLevels, 3, 3>();
      float m[C];  // lane c: row c of L
#pragma unroll
      for (int s4 = 0; s4 < C; s4 += 4) {
        const f4 lr = lds4(&Lrs[c * LT + s4]);
#pragma unroll
        for (int e = 0; e < 4; ++e) m[s4 + e] = lr[e];
      }
      const float dl = Lrs[c * LT + c];  // L_cc
      float wn2 = 0.0f;
#pragma unroll
      for (int ww = 0; ww < NW; ++ww) wn2 += wn2p[ww][c];
      // hardware reciprocal and square root (1 ulp): c_t only scales the write direction
      const float rdl = __builtin_amdgcn_rcpf(dl);
      const float an = __builtin_amdgcn_sqrtf(wn2) * rdl;                // ||A_t k^_t|| = ||w_t|| / L_tt
      const float cs = rdl * __builtin_amdgcn_rcpf(fmaxf(an, eps));      // alpha^_t = c_t w_t
      if (g == 0) cvec[c] = -cs;  // the residual tiles carry -E, see below
      // Z = (I + strict_lower(L) diag(c))^{-1}: lane c holds column c (rows of L live in lanes 0-31)
      float nm[C], Zr[C];
      float ncs = -cs;
      asm volatile("s_nop 1" : "+v"(ncs));   // a DPP read of a VGPR needs 2 wait states after its write
      scale_cols<0>(m, nm, ncs);             // lane t: -L[t][s] c_s
      asm volatile("s_nop 1" : "+v"(nm[0]));
      z_rows<0>(nm, Zr, cc);
      if (g == 0) {
#pragma unroll
        for (int t = 0; t < C; ++t) Zs[t * LT + c] = Zr[t];
      }
      // H = L^{-1} GQ (one MFMA tile), NQ[s][t] = c_s H[s][t] for s <= t
      f4 hq = f4{0, 0, 0, 0};
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float gqv = 0.0f;
#pragma unroll
        for (int ww = 0; ww < NW; ++ww) gqv += Gp[ww][1][(4 * g + r) * LT + c];
        hq = mfma16(la[r], gqv, hq);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int s = 4 * g + r;
        const float csr = __shfl(cs, s);
        NQs[c * LT + s] = (s <= c) ? -(csr * hq[r]) : 0.0f;
      }
      prio<kLevels, 1, 0>();
    }
    __syncthreads();  // (5) Z, NQ, c visible

    // ================= -E^T = Z (-F^T), R^T = Q S0^T, O^T = R^T + (-NQ^T)(-E^T), store o;
    // ce = (-c) (-E^T) = diag(c) E^T
    f4 ce[NJV];
    {
      const f4 za = lds4(&Zs[c * LT + 4 * g]);
#pragma unroll
      for (int jn = 0; jn < NJV; ++jn) {
        f4 et = f4{0, 0, 0, 0};
#pragma unroll
        for (int r = 0; r < 4; ++r) et = mfma16(za[r], ft[jn][r], et);
        ft[jn] = et;
      }
      if (w == sw) r_pass();
      const f4 nqa = lds4(&NQs[c * LT + 4 * g]);
      const f4 cg = lds4(&cvec[4 * g]);
#pragma unroll
      for (int jn = 0; jn < NJV; ++jn) {
#pragma unroll
        for (int r = 0; r < 4; ++r) ot[jn] = mfma16(nqa[r], ft[jn][r], ot[jn]);
        ce[jn] = ft[jn] * cg;
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int t = t0 + 4 * g + r;
        if (t < T) {
          const unsigned ooff = static_cast<unsigned>(t * DV + vcol);
          if constexpr (kEven) {
#pragma unroll
            for (int jn = 0; jn + 1 < NJV; jn += 2)
              io_store2(oh + ooff + 16 * jn, oh + ooff + 16 * jn + 16, ot[jn][r], ot[jn + 1][r]);
            if (NJV % 2 == 1) io_store(oh + ooff + 16 * (NJV - 1), ot[NJV - 1][r]);
          } else {
#pragma unroll
            for (int jn = 0; jn < NJV; ++jn)
              if (owns(jn)) io_store(oh + ooff + (s_row(jn) - s_row(0)), ot[jn][r]);
          }
        }
      }
    }
    // ================= S^T += W diag(c) E^T  (and A -= W W^T on the wave that formed Z)
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const f4 wa = lds4(&Wb[(16 * b + c) * LT + 4 * g]);
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int jn = 0; jn < NJV; ++jn) St[b][jn] = mfma16(wa[r], ce[jn][r], St[b][jn]);
    }
    if (w == sw2) update_A();
  }

  // ---- final state
  {
    float* AT = a.A_T ? a.A_T + static_cast<size_t>(head) * D * D : nullptr;
    float* ST = a.S_T ? a.S_T + static_cast<size_t>(head) * DV * D : nullptr;
    int g2 = g, c2 = c;
    asm volatile("" : "+v"(g2), "+v"(c2));  // recompute the addresses here instead of carrying them over the loop
    const int arc = (4 * g2) * D + col0 + c2;
    const int src = c2 * D + 4 * g2;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      if (AT) {
#pragma unroll
        for (int jn = 0; jn < NJ; ++jn)
#pragma unroll
          for (int r = 0; r < 4; ++r) AT[arc + (16 * b + r) * D + 16 * jn] = At[b][jn][r];
      }
      if (ST) {
#pragma unroll
        for (int jn = 0; jn < NJV; ++jn)
          if (owns(jn))
            *reinterpret_cast<float4*>(ST + src + s_row(jn) * D + 16 * b) =
                make_float4(St[b][jn][0], St[b][jn][1], St[b][jn][2], St[b][jn][3]);
      }
    }
  }
}

template <int D, int DV, int NW, typename IO>
hipError_t launch(const ForwardArgs& a, hipStream_t stream) {
  ForwardArgs args = a;
  void* params[] = {&args};
  const void* fn = a.feature_map ? reinterpret_cast<const void*>(&chunk_kernel<D, DV, NW, IO, true>)
                                 : reinterpret_cast<const void*>(&chunk_kernel<D, DV, NW, IO, false>);
  return hipLaunchKernel(fn, dim3(a.n_heads), dim3(64 * NW), params, 0, stream);
}
template <int D, int DV, int NW>
hipError_t launch_io(const ForwardArgs& a, int io_dtype, hipStream_t stream) {
  return io_dtype == 1 ? launch<D, DV, NW, uint16_t>(a, stream) : launch<D, DV, NW, float>(a, stream);
}

}  // namespace

bool chunk_supported(int d) { return d == 16 || d == 32 || d == 64 || d == 96 || d == 128; }

// Several heads per workgroup (vla_chunk_multihead.hip) or one?  Measured on one MI355X, T = 8192:
//   d = 64 (two-wave workgroups here, four-wave ones of two heads there; both hold 1024 heads per chip at a
//   time): up to 256 heads one workgroup per compute unit either way, 2.5 against 2.7 ms; 257-512 heads 4.1
//   against 2.7 ms (two two-wave workgroups on a compute unit are placed on three of its four SIMDs); 768-1024
//   heads 4.3-4.5 against 4.1-4.2 ms; 2048 heads 8.9 against 8.3 ms, 3072: 13.2 against 12.4, 4096: 17.6 against
//   16.5; but 1280-1536 heads 7.0 against 8.4-8.5 ms: the larger workgroups refill a draining chip two to a
//   compute unit, so a launch that is not a whole number of full rounds pays for its tail.
//   d = 32 (one-wave workgroups here, four heads per workgroup there): up to 1024 heads 2.3 against 2.4 ms,
//   1280-1536 heads 3.35 against 3.25 ms, 2048 heads 4.6 against 3.25 ms, 4096: 9.2 against 6.5.
bool prefer_multihead(int d, int n_heads) {
  if (d == 32) return n_heads > 1024;
  if (d == 64) {
    const int wgs = (n_heads + 1) / 2;
    return n_heads > 256 && (wgs <= 512 || wgs % 512 == 0 || wgs >= 4096);
  }
  return false;
}

// The d_k / 32 waves of a head (one below d_k = 32) share out the d_v / 16 row tiles of S, evenly where the counts
// divide and one by one in turn where they do not: every pair of head sizes runs.
bool chunk_supported(int d_k, int d_v) { return chunk_supported(d_k) && chunk_supported(d_v); }

hipError_t launch_chunk(const ForwardArgs& a, int d_k, int d_v, int io_dtype, hipStream_t stream) {
  if (d_k == d_v && prefer_multihead(d_k, a.n_heads)) return launch_chunk_multihead(a, d_k, io_dtype, stream);
  switch (d_k * 1000 + d_v) {
    case 16016: return launch_io<16, 16, 1>(a, io_dtype, stream);
    case 32032: return launch_io<32, 32, 1>(a, io_dtype, stream);
    case 64064: return launch_io<64, 64, 2>(a, io_dtype, stream);
    case 96096: return launch_io<96, 96, 3>(a, io_dtype, stream);
    case 128128: return launch_io<128, 128, 4>(a, io_dtype, stream);
    case 16032: return launch_io<16, 32, 1>(a, io_dtype, stream);
    case 32016: return launch_io<32, 16, 1>(a, io_dtype, stream);
    case 32064: return launch_io<32, 64, 1>(a, io_dtype, stream);
    case 64032: return launch_io<64, 32, 2>(a, io_dtype, stream);
    case 64128: return launch_io<64, 128, 2>(a, io_dtype, stream);
    case 128064: return launch_io<128, 64, 4>(a, io_dtype, stream);
    case 16064: return launch_io<16, 64, 1>(a, io_dtype, stream);
    case 16096: return launch_io<16, 96, 1>(a, io_dtype, stream);
    case 16128: return launch_io<16, 128, 1>(a, io_dtype, stream);
    case 32096: return launch_io<32, 96, 1>(a, io_dtype, stream);
    case 32128: return launch_io<32, 128, 1>(a, io_dtype, stream);
    case 64096: return launch_io<64, 96, 2>(a, io_dtype, stream);
    case 64016: return launch_io<64, 16, 2>(a, io_dtype, stream);
    case 96016: return launch_io<96, 16, 3>(a, io_dtype, stream);
    case 96032: return launch_io<96, 32, 3>(a, io_dtype, stream);
    case 96064: return launch_io<96, 64, 3>(a, io_dtype, stream);
    case 96128: return launch_io<96, 128, 3>(a, io_dtype, stream);
    case 128016: return launch_io<128, 16, 4>(a, io_dtype, stream);
    case 128032: return launch_io<128, 32, 4>(a, io_dtype, stream);
    case 128096: return launch_io<128, 96, 4>(a, io_dtype, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace vla
