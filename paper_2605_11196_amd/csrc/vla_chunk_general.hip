// Block form of the VLA recurrence with the optional lines of Algorithm 1 (paper, pseudocode appendix) on
// FP32 MFMA: a penalty direction u_t supplied separately from the key (eq. (penalty)), the periodic identity
// refresh A += eta I, the normalised read-out of eq. (output) with its running key sum, and the ELU+1
// feature map on q and k (Section 3.3).
//
// Within a block of at most C = 16 tokens (rows = tokens), entering state A0 (symmetric), S0:
//
//   Y^T = U A0 ,  X^T = K^ A0                        (C x d)   z and A0 k^ before the in-block corrections
//   G = Y^T U^T = L L^T - I                          (C x C)   L_tt^2 = delta_t
//   W^T = L^{-1} Y^T                                 (C x d)   A_t = A0 - sum_{s<=t} w_s w_s^T   (eq. (sm))
//   Hm = L^{-1} (Y^T K^^T)                           (C x C)   Hm[s][t] = w_s . k^_t
//   alpha_t = x_t - sum_{s<=t} Hm[s][t] w_s                    = A_t k^_t          (post-update A)
//   c_t = 1 / max(||alpha_t||, eps)                            alpha^_t = c_t alpha_t
//   P[s][t] = alpha_s . k^_t = (X^T K^^T)[s][t] - sum_{r<=s} Hm[r][s] Hm[r][t]
//   AQ[s][t] = alpha_s . q_t = (X^T Q^T)[s][t] - sum_{r<=s} Hm[r][s] (L^{-1} Y^T Q^T)[r][t]
//   F^T = V - K^ S0^T ,  E^T = Z F^T ,  Z = (I + N)^{-1},  N[t][s] = c_s P[s][t] for s < t    (eq. (s-update))
//   O^T = Q S0^T + NQ^T E^T ,  NQ[s][t] = c_s AQ[s][t] for s <= t, else 0
//   S1^T = S0^T + Alpha diag(c) E^T ,  A1 = A0 - W W^T
//
// With u = k^ and no refresh the rows of X and Y coincide and this reduces to the block form of the plain
// kernel (template flag FULL = false: one sweep of A, two Gram matrices).
//
// Identity refresh: a step whose 1-based index is a multiple of the period adds eta I to A after the
// rank-1 update and before the write direction is formed, anywhere inside a block.  With n_t the number of
// refresh steps among the block's tokens before t and n'_t = n_{t+1} (before or at t), token t updates with
// A0 + eta n_t I - sum_{r<t} w_r w_r^T and writes with A0 + eta n'_t I - sum_{r<=t} w_r w_r^T, so everything
// above holds with
//   y'_t = y_t + eta n_t u_t ,   x'_t = x_t + eta n'_t k^_t
// in place of y_t, x_t (the Gram matrices are formed from Y', X'), with the matrix to factor taken as
// I + u_s . y'_t for t <= s (the upper triangle of Y' U^T, mirrored: the base matrix of the earlier token
// counts), and A1 = A0 + eta n_C I - W W^T.
//
// Normalised read-out: o_t is divided by max(q_t . zkey_t, eps), zkey_t = zkey_0 + sum_{s<=t} k_s with k_s
// the key as used before L2 normalisation, k_s = max(||k_s||, eps) k^_s; inside a block
// q_t . zkey_t = q_t . zkey_start + sum_{s<=t} ||k_s|| (Q K^^T)[t][s].
//
// Work split: D/16 waves per (batch, head); wave w owns columns [16w, 16w+16) of A and the same rows of S
// (with a value head size other than D: the row tiles w, w + D/16, ... of S) as 16x16 MFMA accumulator tiles
// resident in VGPRs for the whole sequence.  The C x C Gram matrices are
// shared out over the waves (each one contracts over the whole head dimension), the C x C factorisations
// run on one wave each, rotating with the block index.
//
// v_mfma_f32_16x16x4_f32 register layout, lane l = 16*g + c:
//   A operand: A[m = c][k = g]      B operand: B[k = g][n = c]      C/D: reg r -> D[m = 4g + r][n = c]
#include "vla_mfma_util.h"

namespace vla {
namespace {

// C x C Gram matrices of a block, [m][n] = sum_j left[m][j] right[n][j]
enum GramTile {
  kG = 0,   // Y U^T
  kGK,      // Y K^^T
  kGQ,      // Y Q^T
  kGX,      // X K^^T
  kXQ,      // X Q^T
  kQK,      // Q K^^T      (normalised read-out)
  kQZ,      // Q zkey^T    (normalised read-out; only column 0 is populated)
  kNumGram
};

// FULL: Y and X differ (a separate u, or a refresh period): two sweeps of A and five Gram matrices.
// SCAN: phase 1 of the two-phase and time-parallel modes: one workgroup per (head, time segment) runs the A
//       chain only, from the A the segment starts with, and writes what the S recurrence needs into the
//       workspace (the layout of vla_mfma_util.h: 1 / ||k_t||, the write directions alpha_t in W's place, Z,
//       -NQ^T, -c_t and the reciprocal read-out denominators); S, v and o are not touched.
// DV: head size of v and o (rows of S).  The DV / 16 row tiles of S go to the waves in turn (tile t to wave
//     t % NW: exactly one each for square heads); a wave with fewer tiles than the others, or none, runs its spare
//     slots on a copy of the last tile and stores nothing from them.
template <int D, int DV, typename IO, bool FULL, bool SCAN>
__global__ void __launch_bounds__(4 * D, (SCAN && D <= 64) ? 3 : 1) chunk_general_kernel(ForwardArgs a) {
  constexpr int NW = D / 16;       // waves; wave w owns columns 16w..16w+15
  constexpr int TV = DV / 16;      // row tiles of S
  constexpr int NJV = (TV + NW - 1) / NW;   // tile slots per wave
  static_assert(DV % 16 == 0 && (!SCAN || DV == D), "whole tiles of S");
  constexpr int NB = D / 16;       // 16-row blocks over the head dimension
  constexpr int LD = D + 4;        // row stride of the token-major LDS arrays
  // Staging: a token row is split over thread slots of EPT elements.  At the power-of-two head sizes every
  // thread stages 4 elements; at d = 96 a row takes 12 threads of 8 elements in a group of 16 (the other four
  // lanes of the group and the last two waves stage nothing), so that a row sums with a power-of-two shuffle.
  constexpr bool PADDED = (D & (D - 1)) != 0;
  constexpr int EPT = PADDED ? 8 : 4;           // staged elements per thread per tensor
  constexpr int TPR = PADDED ? 16 : D / EPT;    // thread slots per token row (inside one wave)
  static_assert(D % EPT == 0 && D / EPT <= TPR && C * TPR <= 4 * D, "staging layout");
  constexpr int UROWS = FULL ? C : 1;
  // Y = X: the Gram matrices that differ only in u against k^ coincide
  constexpr int iGK = FULL ? kGK : kG;
  constexpr int iGX = FULL ? kGX : kG;
  constexpr int iXQ = FULL ? kXQ : kGQ;

  __shared__ __align__(16) float Ksb[2][C * LD];      // K^  [t][j], double-buffered over blocks
  __shared__ __align__(16) float Qsb[2][C * LD];      // Q   [t][j]
  __shared__ __align__(16) float Usb[UROWS * LD];     // U   [t][j] (dead after the Gram phase of its block)
  __shared__ __align__(16) float Ys[C * LD];          // Y^T [t][j]
  __shared__ __align__(16) float Xsb[UROWS * LD];     // X^T [t][j]
  __shared__ __align__(16) float Wb[D * LT];          // W     [j][t]
  __shared__ __align__(16) float Ab[D * LT];          // Alpha [j][t]
  __shared__ __align__(16) float Gs[kNumGram][C * LT];
  __shared__ __align__(16) float Lis[C * LT];         // L^{-1} [t][s]
  __shared__ __align__(16) float Ps[C * LT];          // P transposed: [t][s] = alpha_s . k^_t
  __shared__ __align__(16) float Zs[C * LT];          // Z   [t][s]
  __shared__ __align__(16) float NQs[C * LT];         // -NQ^T [t][s]
  __shared__ __align__(16) float wn2p[NW][C];         // per-wave partial ||alpha_t||^2
  __shared__ __align__(16) float cvec[C];             // -c_t
  __shared__ __align__(16) float rdens[C];            // 1 / max(q_t . zkey_t, eps)
  __shared__ __align__(16) float nks[2][C];           // max(||k_t||, eps), double-buffered with K^
  __shared__ __align__(16) float zks[D];              // running key sum (each wave touches its own columns)
  __shared__ __align__(16) float ens[2][C + 4];       // eta n_i, i = 0..C: refresh steps among a block's first i tokens

  const int head = SCAN ? blockIdx.x / a.n_seg : blockIdx.x;
  const int seg = SCAN ? blockIdx.x - head * a.n_seg : 0;
  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int c = lane & 15;
  const int g = lane >> 4;
  const int tb = SCAN ? seg * a.seg_blocks * C : 0;                 // first token of this workgroup's range
  const int T = SCAN ? min(a.T, tb + a.seg_blocks * C) : a.T;       // one past its last token
  const float eps = a.eps;
  const int col0 = 16 * w;
  const int period = a.refresh_period;
  const float eta = a.refresh_eta;
  const bool norm_out = a.normalise_output != 0;
  const bool key_sum = norm_out || a.zkey_T != nullptr;
  const bool fmap = a.feature_map != 0;
  const bool has_u = a.u != nullptr;
  const float* Us = FULL ? Usb : nullptr;   // set per block when Y = X
  const float* Xs = FULL ? Xsb : Ys;

  // first S row of this wave's tile slot jn, and whether the slot holds a tile of its own
  auto s_row = [&](int jn) -> int {
    const int t = w + NW * jn;
    return 16 * (t < TV ? t : TV - 1);
  };
  auto owns = [&](int jn) -> bool { return w + NW * jn < TV; };
  // ---- resident state: At[b][r] = A[16b + 4g + r][col0 + c],  St[jn][b][r] = S[s_row(jn) + c][16b + 4g + r]
  f4 At[NB], St[NJV][NB];
  {
    const float* A0 = (SCAN && a.seg_A) ? a.seg_A + static_cast<size_t>(blockIdx.x) * D * D
                                        : (a.A0 ? a.A0 + static_cast<size_t>(head) * D * D : nullptr);
    const float* S0 = (!SCAN && a.S0) ? a.S0 + static_cast<size_t>(head) * DV * D : nullptr;
    const float diag = 1.0f / a.lambda0;
    const int arc = (4 * g) * D + col0 + c;
    const int src = c * D + 4 * g;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      if (A0) {
#pragma unroll
        for (int r = 0; r < 4; ++r) At[b][r] = A0[arc + (16 * b + r) * D];
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) At[b][r] = (16 * b + 4 * g + r == col0 + c) ? diag : 0.0f;
      }
#pragma unroll
      for (int jn = 0; jn < NJV; ++jn) {
        if (S0) {
          const float4 x = *reinterpret_cast<const float4*>(S0 + src + s_row(jn) * D + 16 * b);
          St[jn][b] = f4{x.x, x.y, x.z, x.w};
        } else {
          St[jn][b] = f4{0, 0, 0, 0};
        }
      }
    }
  }
  if (lane < 16) {   // key sum entering this range: the caller's, or the one the segment starts with
    const float* z0 = (SCAN && a.seg_zkey) ? a.seg_zkey + static_cast<size_t>(blockIdx.x) * D
                                           : (a.zkey0 ? a.zkey0 + static_cast<size_t>(head) * D : nullptr);
    zks[col0 + lane] = z0 ? z0[col0 + lane] : 0.0f;
  }
  // workspace records of this head (SCAN)
  const int nblk_all = (a.T + C - 1) / C;
  float* wsh = SCAN ? a.ws + static_cast<size_t>(head) * head_stride(nblk_all, D) : nullptr;
  float* RN = SCAN ? wsh + off_rn(nblk_all, D) : nullptr;
  float* WT = SCAN ? wsh + off_wt(nblk_all, D) : nullptr;
  float* SMp = SCAN ? wsh + off_sm(nblk_all, D) : nullptr;

  const size_t slab = static_cast<size_t>(head) * static_cast<size_t>(a.T) * D;
  const IO* qh = static_cast<const IO*>(a.q) + slab;
  const IO* kh = static_cast<const IO*>(a.k) + slab;
  const size_t slab_v = static_cast<size_t>(head) * static_cast<size_t>(a.T) * DV;
  const IO* vh = static_cast<const IO*>(a.v) + slab_v;
  const IO* uh = has_u ? static_cast<const IO*>(a.u) + slab : kh;
  IO* oh = static_cast<IO*>(a.o) + slab_v;

  // staging role of this thread: token row and 4-element column segment
  const int srow = tid / TPR;
  const int sseg = (tid % TPR) * EPT;
  const bool stager = !PADDED || (tid < C * TPR && sseg < D);   // this thread holds a row segment
  const bool stage_wave = !PADDED || tid < C * TPR;             // uniform per wave

  RawRow<IO, EPT> kpre, qpre, upre;
  IO vpre[NJV][4];  // V in accumulator layout: V[t0 + 4g + r][s_row(jn) + c]

  // Loads never branch on the row: rows past the end read the last valid row and are zeroed when consumed.
  auto load_kqu = [&](int t0) {
    if (stager) {
      const int tr = t0 + srow;
      const unsigned off = static_cast<unsigned>((tr < T ? tr : T - 1) * D + sseg);
      kpre.load(kh + off);
      qpre.load(qh + off);
      if (has_u) upre.load(uh + off);
    }
  };
  auto load_v = [&](int t0) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int t = t0 + 4 * g + r;
      const unsigned voff = static_cast<unsigned>((t < T ? t : T - 1) * DV + c);
#pragma unroll
      for (int jn = 0; jn < NJV; ++jn) vpre[jn][r] = vh[voff + s_row(jn)];
    }
  };
  auto row_total = [&](float x) -> float {
#pragma unroll
    for (int off = TPR / 2; off >= 1; off >>= 1) x += __shfl_xor(x, off);
    return x;
  };
  // 1 / max(sqrt(ss), eps): hardware reciprocal square root refined by one Newton step
  auto inv_norm = [&](float ss, float& clamped) -> float {
    clamped = fmaxf(ss, eps * eps);
    const float rn = __builtin_amdgcn_rsqf(clamped);
    return rn * fmaf(-0.5f * clamped * rn, rn, 1.5f);
  };
  // this thread's share of the block of `len` live tokens that starts at token tfirst (step index idx0, 1-based,
  // counted over the whole sequence): K^, Q (and U) into LDS half `buf`, and the refresh counts of the block
  auto stage = [&](int len, int idx0, int buf, int tfirst) {
    if (!stage_wave) return;
    const bool live = srow < len && stager;
    float x[EPT], kn[EPT];
    if (stager) {
      kpre.unpack(x);
    } else {
#pragma unroll
      for (int e = 0; e < EPT; ++e) x[e] = 0.0f;
    }
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      if (fmap) x[e] = elu_plus_one(x[e]);
      x[e] = live ? x[e] : 0.0f;
    }
    float ss = 0.0f;
#pragma unroll
    for (int e = 0; e < EPT; ++e) ss = fmaf(x[e], x[e], ss);
    float sm;
    const float rn = inv_norm(row_total(ss), sm);
#pragma unroll
    for (int e = 0; e < EPT; ++e) kn[e] = x[e] * rn;
    float us[EPT];
    float su = 0.0f;
    if constexpr (FULL) {
      if (has_u) {
        if (stager) {
          upre.unpack(us);
        } else {
#pragma unroll
          for (int e = 0; e < EPT; ++e) us[e] = 0.0f;
        }
#pragma unroll
        for (int e = 0; e < EPT; ++e) us[e] = live ? us[e] : 0.0f;
        float uu = 0.0f;
#pragma unroll
        for (int e = 0; e < EPT; ++e) uu = fmaf(us[e], us[e], uu);
        float um;
        su = a.u_scale * inv_norm(row_total(uu), um);
      }
      if (tid <= C) {  // multiples of the period among the step indices idx0 .. idx0 + tid - 1
        const int n = period > 0 ? (idx0 - 1 + tid) / period - (idx0 - 1) / period : 0;
        ens[buf][tid] = eta * static_cast<float>(n);
      }
    }
    if (!stager) return;
#pragma unroll
    for (int e = 0; e < EPT; e += 4) {
      *reinterpret_cast<f4*>(&Ksb[buf][srow * LD + sseg + e]) = f4{kn[e], kn[e + 1], kn[e + 2], kn[e + 3]};
    }
    if (sseg == 0) {
      nks[buf][srow] = sm * rn;  // max(||k||, eps)
      if constexpr (SCAN) RN[tfirst + srow] = live ? rn : 0.0f;   // rows past the end: zero keys
    }
    qpre.unpack(x);
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      if (fmap) x[e] = elu_plus_one(x[e]);
      x[e] = live ? x[e] : 0.0f;
    }
#pragma unroll
    for (int e = 0; e < EPT; e += 4) {
      *reinterpret_cast<f4*>(&Qsb[buf][srow * LD + sseg + e]) = f4{x[e], x[e + 1], x[e + 2], x[e + 3]};
    }
    if constexpr (FULL) {
#pragma unroll
      for (int e = 0; e < EPT; e += 4) {
        *reinterpret_cast<f4*>(&Usb[srow * LD + sseg + e]) =
            has_u ? f4{us[e] * su, us[e + 1] * su, us[e + 2] * su, us[e + 3] * su}
                  : f4{kn[e], kn[e + 1], kn[e + 2], kn[e + 3]};   // u = k^ without a separate direction
      }
    }
  };

  if (tb < T) {
    load_kqu(tb);
    if constexpr (!SCAN) load_v(tb);
    stage(T - tb < C ? T - tb : C, a.step_offset + tb + 1, 0, tb);
    if (tb + C < T) load_kqu(tb + C);
  }
  __syncthreads();  // first block staged, zks initialised

  int blk = 0;
  for (int t0 = tb; t0 < T; t0 += C, ++blk) {
    const float* Ks = Ksb[blk & 1];
    const float* Qs = Qsb[blk & 1];
    const float* en = ens[blk & 1];
    if constexpr (!FULL) Us = Ks;
    const int len = T - t0 < C ? T - t0 : C;
    const int tn = t0 + C;                           // start of the next block
    auto stage_next = [&]() {
      if (tn < T) {
        stage(T - tn < C ? T - tn : C, a.step_offset + tn + 1, (blk + 1) & 1, tn);
        if (tn + C < T) load_kqu(tn + C);
      }
    };
    int cc = c;  // opaque copy: keeps lane-dependent masks from being hoisted out of the loop
    asm volatile("" : "+v"(cc));

    f4 ft[NJV];  // starts as -V^T, becomes -F^T = K^ S0^T - V^T
#pragma unroll
    for (int jn = 0; jn < NJV; ++jn) ft[jn] = f4{0, 0, 0, 0};
    if constexpr (!SCAN) {
#pragma unroll
      for (int jn = 0; jn < NJV; ++jn)
#pragma unroll
        for (int r = 0; r < 4; ++r) ft[jn][r] = (4 * g + r < len) ? neg_widen(vpre[jn][r]) : 0.0f;
      if (tn < T) load_v(tn);
    }

    // ================= Y^T = U A0, X^T = K^ A0 (this wave's columns) -> LDS;  -F^T = K^ S0^T - V^T
    f4 yt = f4{0, 0, 0, 0}, xt = f4{0, 0, 0, 0};
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const f4 ka = lds4(&Ks[c * LD + 16 * b + 4 * g]);
      if constexpr (FULL) {
        const f4 ua = lds4(&Us[c * LD + 16 * b + 4 * g]);
#pragma unroll
        for (int r = 0; r < 4; ++r) yt = mfma16(ua[r], At[b][r], yt);
#pragma unroll
        for (int r = 0; r < 4; ++r) xt = mfma16(ka[r], At[b][r], xt);
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) yt = mfma16(ka[r], At[b][r], yt);
      }
      if constexpr (!SCAN) {
#pragma unroll
        for (int jn = 0; jn < NJV; ++jn)
#pragma unroll
          for (int r = 0; r < 4; ++r) ft[jn] = mfma16(ka[r], St[jn][b][r], ft[jn]);
      }
    }
    if constexpr (FULL) {
      if (period > 0) {  // y'_t = y_t + eta n_t u_t,  x'_t = x_t + eta n'_t k^_t  (n'_t = n_{t+1})
        const f4 e0 = lds4(&en[4 * g]);
        const f4 e1 = f4{e0[1], e0[2], e0[3], en[4 * g + 4]};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          yt[r] = fmaf(e0[r], Us[(4 * g + r) * LD + col0 + c], yt[r]);
          xt[r] = fmaf(e1[r], Ks[(4 * g + r) * LD + col0 + c], xt[r]);
        }
      }
    } else {
      xt = yt;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      Ys[(4 * g + r) * LD + col0 + c] = yt[r];
      if constexpr (FULL) Xsb[(4 * g + r) * LD + col0 + c] = xt[r];
    }
    __syncthreads();  // (1) Y^T, X^T complete

    // ================= Gram matrices, shared out over the waves
    {
      int slot = 0;
#pragma unroll
      for (int i = 0; i < kNumGram; ++i) {
        if (!FULL && (i == kGK || i == kGX || i == kXQ)) continue;
        if ((i == kQK || i == kQZ) && !norm_out) continue;
        const bool mine = (slot % NW) == w;
        ++slot;
        if (!mine) continue;
        const float* left = (i == kG || i == kGK || i == kGQ) ? Ys : (i == kGX || i == kXQ) ? Xs : Qs;
        const float* right = (i == kG) ? Us : (i == kGK || i == kGX || i == kQK) ? Ks : Qs;
        f4 acc0 = f4{0, 0, 0, 0}, acc1 = f4{0, 0, 0, 0};  // two chains: the tile is one wave's whole job here
#pragma unroll
        for (int b = 0; b < NB; ++b) {
          const f4 av = lds4(&left[c * LD + 16 * b + 4 * g]);
          f4 bv;
          if (i == kQZ) {
            const f4 zv = lds4(&zks[16 * b + 4 * g]);
            bv = (cc == 0) ? zv : f4{0, 0, 0, 0};
          } else {
            bv = lds4(&right[c * LD + 16 * b + 4 * g]);
          }
          acc0 = mfma16(av[0], bv[0], acc0);
          acc1 = mfma16(av[1], bv[1], acc1);
          acc0 = mfma16(av[2], bv[2], acc0);
          acc1 = mfma16(av[3], bv[3], acc1);
        }
        acc0 += acc1;
#pragma unroll
        for (int r = 0; r < 4; ++r) Gs[i][(4 * g + r) * LT + c] = acc0[r];
      }
    }
    __syncthreads();  // (2) Gram matrices visible

    // ================= phase 1 (one wave): Cholesky of I + G and L^{-1}
    const int sw = (blk + head) % NW;
    const int sw2 = (sw + (NW > 2 ? NW / 2 + 1 : 1)) % NW;  // another wave, on another SIMD, forms c, Z, NQ
    f4 ot[NJV];  // R^T = Q S0^T, later O^T
    auto r_pass = [&]() {
#pragma unroll
      for (int jn = 0; jn < NJV; ++jn) ot[jn] = f4{0, 0, 0, 0};
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const f4 qa = lds4(&Qs[c * LD + 16 * b + 4 * g]);
#pragma unroll
        for (int jn = 0; jn < NJV; ++jn)
#pragma unroll
          for (int r = 0; r < 4; ++r) ot[jn] = mfma16(qa[r], St[jn][b][r], ot[jn]);
      }
    };
    if (w != sw) {
      if constexpr (!SCAN) r_pass();
      stage_next();
    } else {
      // Lanes 0-31 hold rows of I + G (-> rows of L), lanes 32-63 columns of the identity (-> columns of
      // L^{-1}); one broadcast of L[j][t] serves the trailing update and the forward substitution.
      __builtin_amdgcn_s_setprio(3);   // the dependent chain is what the other waves wait for: issue it first
      float m[C];
      const bool lower = lane < 32;
#pragma unroll
      for (int s4 = 0; s4 < C; s4 += 4) {
        f4 acc = lds4(&Gs[kG][c * LT + s4]);
        if (FULL && period > 0) {  // entry (c, s) with s < c from its mirror image (s, c): see the header
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float mir = Gs[kG][(s4 + e) * LT + c];
            acc[e] = (s4 + e < cc) ? mir : acc[e];
          }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) m[s4 + e] = (lower ? acc[e] : 0.0f) + ((s4 + e) == cc ? 1.0f : 0.0f);
      }
#pragma unroll
      for (int t = 0; t < C; ++t) {
        const float p = readlane(m[t], t);  // pivot = delta_t >= 1
        const float ri = __builtin_amdgcn_rsqf(p);
        const float li = m[t] * ri;  // lanes <32: column t of L;  lanes >=32: row t of L^{-1}, final
        m[t] = li;
#pragma unroll
        for (int j = t + 1; j < C; ++j) m[j] = fmaf(-li, readlane(li, j), m[j]);
      }
      if (g == 2) {
#pragma unroll
        for (int t = 0; t < C; ++t) Lis[t * LT + c] = m[t];
      }
      __builtin_amdgcn_s_setprio(0);
    }
    __syncthreads();  // (3) L^{-1} visible

    // ================= W^T = L^{-1} Y^T,  Hm = L^{-1} (Y K^^T),  Alpha^T = X^T - M W^T,  ||alpha_t||^2
    const f4 la = lds4(&Lis[c * LT + 4 * g]);
    f4 nwt;   // -W^T tile
    f4 mop;   // M as an A operand: M[t = c][s = 4g + r] = Hm[s][t] for s <= t
    f4 nhm;   // -Hm in accumulator layout
    {
      f4 acc = f4{0, 0, 0, 0};
      f4 hm = f4{0, 0, 0, 0};
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        acc = mfma16(la[r], yt[r], acc);
        hm = mfma16(la[r], Gs[iGK][(4 * g + r) * LT + c], hm);
      }
      nwt = -acc;
      nhm = -hm;
      *reinterpret_cast<f4*>(&Wb[(col0 + c) * LT + 4 * g]) = acc;
#pragma unroll
      for (int r = 0; r < 4; ++r) mop[r] = (4 * g + r <= cc) ? hm[r] : 0.0f;
      f4 at = xt;
#pragma unroll
      for (int r = 0; r < 4; ++r) at = mfma16(mop[r], nwt[r], at);
      f4 n2 = at * at;
#pragma unroll
      for (int r = 0; r < 4; ++r) n2[r] = row_sum16(n2[r]);
      if (c == 0) *reinterpret_cast<f4*>(&wn2p[w][4 * g]) = n2;
      if constexpr (SCAN) {
        *reinterpret_cast<f4*>(WT + (static_cast<size_t>(t0 / C) * D + col0 + c) * C + 4 * g) = at;
      } else {
        *reinterpret_cast<f4*>(&Ab[(col0 + c) * LT + 4 * g]) = at;
      }
    }
    __syncthreads();  // (4) W, Alpha and the norm partials visible

    // ================= phase 2 (wave sw2): c_t, Z, NQ, read-out denominators -- the others update A
    auto update_A = [&]() {
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const f4 wa = lds4(&Wb[(16 * b + c) * LT + 4 * g]);
#pragma unroll
        for (int r = 0; r < 4; ++r) At[b] = mfma16(wa[r], nwt[r], At[b]);
      }
      if (FULL && period > 0) {  // + eta n on the diagonal (rows 16w + 4g + r against column 16w + c), n counted
        const float en_end = en[len];  // over the live tokens
#pragma unroll
        for (int b = 0; b < NB; ++b) {
          if (b == w) {
#pragma unroll
            for (int r = 0; r < 4; ++r) At[b][r] += (4 * g + r == cc) ? en_end : 0.0f;
          }
        }
      }
    };
    if (w != sw2) update_A();
    if (w == sw) stage_next();
    if (w == sw2) {
      __builtin_amdgcn_s_setprio(3);
      float wn2 = 0.0f;
#pragma unroll
      for (int ww = 0; ww < NW; ++ww) wn2 += wn2p[ww][c];
      const float cs = __builtin_amdgcn_rcpf(fmaxf(__builtin_amdgcn_sqrtf(wn2), eps));  // alpha^_t = c_t alpha_t
      float* smb = SCAN ? SMp + static_cast<size_t>(t0 / C) * SMB : nullptr;   // this block's record
      if (g == 0) {
        if constexpr (SCAN) smb[2 * C * C + c] = -cs;
        else cvec[c] = -cs;
      }
      // P and AQ in accumulator layout [s = 4g + r][t = c]
      f4 pt, aq;
      f4 nhq = f4{0, 0, 0, 0};
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        pt[r] = Gs[iGX][(4 * g + r) * LT + c];
        aq[r] = Gs[iXQ][(4 * g + r) * LT + c];
        nhq = mfma16(-la[r], Gs[kGQ][(4 * g + r) * LT + c], nhq);  // -(L^{-1} Y Q^T)
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        pt = mfma16(mop[r], nhm[r], pt);
        aq = mfma16(mop[r], nhq[r], aq);
      }
      // rows of P^T on lanes: lane t reads alpha_s . k^_t for all s
      *reinterpret_cast<f4*>(&Ps[c * LT + 4 * g]) = pt;
      float m[C];
#pragma unroll
      for (int s4 = 0; s4 < C; s4 += 4) {
        const f4 pr = lds4(&Ps[c * LT + s4]);  // same wave wrote it: LDS operations of one wave are ordered
#pragma unroll
        for (int e = 0; e < 4; ++e) m[s4 + e] = pr[e];
      }
      float nm[C], Zr[C];
      float ncs = -cs;
      asm volatile("s_nop 1" : "+v"(ncs));   // a DPP read of a VGPR needs 2 wait states after its write
      scale_cols<0>(m, nm, ncs);             // lane t: -P[s][t] c_s = -N[t][s]
      asm volatile("s_nop 1" : "+v"(nm[0]));
      z_rows<0>(nm, Zr, cc);
      if (g == 0) {
#pragma unroll
        for (int t = 0; t < C; ++t) {
          if constexpr (SCAN) smb[t * C + c] = Zr[t];
          else Zs[t * LT + c] = Zr[t];
        }
      }
      f4 nq;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int s = 4 * g + r;
        const float csr = __shfl(cs, s);
        nq[r] = (s <= c) ? -(csr * aq[r]) : 0.0f;
        if constexpr (!SCAN) NQs[c * LT + s] = nq[r];
      }
      if constexpr (SCAN) *reinterpret_cast<f4*>(smb + C * C + c * C + 4 * g) = nq;  // -NQ^T[t = c][s = 4g + r]
      if (norm_out) {  // q_t . zkey_t for t = 4g + r: key-sum part + in-block part over s = c <= t
        const float nk = nks[blk & 1][c];
        f4 den;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float qk = Gs[kQK][(4 * g + r) * LT + c];
          const float qz = Gs[kQZ][(4 * g + r) * LT + c];
          den[r] = row_sum16(qz + ((cc <= 4 * g + r) ? qk * nk : 0.0f));
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) den[r] = 1.0f / fmaxf(den[r], eps);
        if (c == 0) {
          if constexpr (SCAN) *reinterpret_cast<f4*>(smb + 2 * C * C + C + 4 * g) = den;
          else *reinterpret_cast<f4*>(&rdens[4 * g]) = den;
        }
      }
      __builtin_amdgcn_s_setprio(0);
    }
    __syncthreads();  // (5) Z, NQ, c, denominators visible; the next block is staged in full

    // ================= -E^T = Z (-F^T), O^T = Q S0^T + (-NQ^T)(-E^T), store o;  ce = diag(c) E^T
    if constexpr (!SCAN) {
    f4 ce[NJV];
    {
      const f4 za = lds4(&Zs[c * LT + 4 * g]);
      f4 et[NJV];
#pragma unroll
      for (int jn = 0; jn < NJV; ++jn) {
        et[jn] = f4{0, 0, 0, 0};
#pragma unroll
        for (int r = 0; r < 4; ++r) et[jn] = mfma16(za[r], ft[jn][r], et[jn]);
      }
      if (w == sw) r_pass();
      const f4 nqa = lds4(&NQs[c * LT + 4 * g]);
      const f4 cg = lds4(&cvec[4 * g]);
#pragma unroll
      for (int jn = 0; jn < NJV; ++jn) {
#pragma unroll
        for (int r = 0; r < 4; ++r) ot[jn] = mfma16(nqa[r], et[jn][r], ot[jn]);
        ce[jn] = et[jn] * cg;
        if (norm_out) ot[jn] *= lds4(&rdens[4 * g]);
        if (owns(jn)) {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            if (4 * g + r < len)
              io_store(oh + static_cast<unsigned>((t0 + 4 * g + r) * DV + s_row(jn) + c), ot[jn][r]);
          }
        }
      }
    }
    // ================= S^T += Alpha diag(c) E^T  (and A -= W W^T on the wave that formed Z)
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const f4 aa = lds4(&Ab[(16 * b + c) * LT + 4 * g]);
#pragma unroll
      for (int jn = 0; jn < NJV; ++jn)
#pragma unroll
        for (int r = 0; r < 4; ++r) St[jn][b] = mfma16(aa[r], ce[jn][r], St[jn][b]);
    }
    }  // !SCAN
    if (w == sw2) update_A();
    if (key_sum && lane < 16) {  // zkey += sum over the block's tokens of ||k_s|| k^_s, this wave's columns
      float zk = zks[col0 + lane];
#pragma unroll
      for (int s = 0; s < C; ++s) zk = fmaf(nks[blk & 1][s], Ks[s * LD + col0 + lane], zk);
      zks[col0 + lane] = zk;
    }
  }

  // ---- final state (SCAN: A and the key sum after the last segment; S belongs to phase 2)
  if (!SCAN || seg == a.n_seg - 1) {
    float* AT = a.A_T ? a.A_T + static_cast<size_t>(head) * D * D : nullptr;
    float* ST = (!SCAN && a.S_T) ? a.S_T + static_cast<size_t>(head) * DV * D : nullptr;
    const int arc = (4 * g) * D + col0 + c;
    const int src = c * D + 4 * g;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      if (AT) {
#pragma unroll
        for (int r = 0; r < 4; ++r) AT[arc + (16 * b + r) * D] = At[b][r];
      }
      if (ST) {
#pragma unroll
        for (int jn = 0; jn < NJV; ++jn)
          if (owns(jn))
            *reinterpret_cast<float4*>(ST + src + s_row(jn) * D + 16 * b) =
                make_float4(St[jn][b][0], St[jn][b][1], St[jn][b][2], St[jn][b][3]);
      }
    }
    if (a.zkey_T != nullptr && lane < 16) {
      a.zkey_T[static_cast<size_t>(head) * D + col0 + lane] = zks[col0 + lane];
    }
  }
}

template <int D, int DV, typename IO>
hipError_t launch(const ForwardArgs& a, hipStream_t stream) {
  ForwardArgs args = a;
  void* params[] = {&args};
  const bool full = a.u != nullptr || a.refresh_period > 0;
  const void* fn = full ? reinterpret_cast<const void*>(&chunk_general_kernel<D, DV, IO, true, false>)
                        : reinterpret_cast<const void*>(&chunk_general_kernel<D, DV, IO, false, false>);
  return hipLaunchKernel(fn, dim3(a.n_heads), dim3(4 * D), params, 0, stream);
}
template <int D, int DV>
hipError_t launch_io(const ForwardArgs& a, int io_dtype, hipStream_t stream) {
  return io_dtype == 1 ? launch<D, DV, uint16_t>(a, stream) : launch<D, DV, float>(a, stream);
}
template <int D>
hipError_t launch_dv(const ForwardArgs& a, int d_v, int io_dtype, hipStream_t stream) {
  switch (d_v) {
    case 16: return launch_io<D, 16>(a, io_dtype, stream);
    case 32: return launch_io<D, 32>(a, io_dtype, stream);
    case 64: return launch_io<D, 64>(a, io_dtype, stream);
    case 96: return launch_io<D, 96>(a, io_dtype, stream);
    case 128: return launch_io<D, 128>(a, io_dtype, stream);
    default: return hipErrorInvalidValue;
  }
}
// phase 1 of the two-phase and time-parallel modes with options: one workgroup per (head, segment)
template <int D, typename IO>
hipError_t launch_scan(const ForwardArgs& a, hipStream_t stream) {
  ForwardArgs args = a;
  void* params[] = {&args};
  const bool full = a.u != nullptr || a.refresh_period > 0;
  const void* fn = full ? reinterpret_cast<const void*>(&chunk_general_kernel<D, D, IO, true, true>)
                        : reinterpret_cast<const void*>(&chunk_general_kernel<D, D, IO, false, true>);
  const long long wgs = static_cast<long long>(a.n_heads) * a.n_seg;
  if (wgs > 0x7fffffffLL) return hipErrorInvalidValue;
  return hipLaunchKernel(fn, dim3(static_cast<unsigned>(wgs)), dim3(4 * D), params, 0, stream);
}

}  // namespace

hipError_t launch_chunk_general(const ForwardArgs& a, int d, int d_v, int io_dtype, hipStream_t stream) {
  switch (d) {
    case 16: return launch_dv<16>(a, d_v, io_dtype, stream);
    case 32: return launch_dv<32>(a, d_v, io_dtype, stream);
    case 64: return launch_dv<64>(a, d_v, io_dtype, stream);
    case 96: return launch_dv<96>(a, d_v, io_dtype, stream);
    case 128: return launch_dv<128>(a, d_v, io_dtype, stream);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_a_scan_general(const ForwardArgs& a, int d, int io_dtype, hipStream_t stream) {
  const bool bf = io_dtype == 1;
  switch (d) {
    case 32: return bf ? launch_scan<32, uint16_t>(a, stream) : launch_scan<32, float>(a, stream);
    case 64: return bf ? launch_scan<64, uint16_t>(a, stream) : launch_scan<64, float>(a, stream);
    case 96: return bf ? launch_scan<96, uint16_t>(a, stream) : launch_scan<96, float>(a, stream);
    case 128: return bf ? launch_scan<128, uint16_t>(a, stream) : launch_scan<128, float>(a, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace vla
