// Two-phase split of the VLA forward recurrence for small B*H (paper Section 3.3 / Algorithm 2's
// premise): the A recurrence never reads S (eq. (sm) uses only u_t), so it can run first and hand the
// S recurrence everything it needs; the rows of S then evolve independently of each other
// (S_t[i,:] = S_{t-1}[i,:] + e_t[i] alpha^_t^T) and are spread over many more workgroups than heads.
//
// Same block form (16 tokens) and notation as vla_chunk.hip.  Per (head, block) the workspace holds
//   RN  [16]         1 / max(||k_t||, eps) per token (0 for rows past the end): the S recurrence re-forms
//                    k^_t = k_t * RN[t] from the raw keys, so the normalised keys never travel through memory
//   W   [D][16]      w_t = z_t / sqrt(delta_t), tokens contiguous
//   SM  [544]        Z | -NQ^T | -c_t | 1 / max(q_t . zkey_t, eps)  (two 16x16 row-major matrices and two vectors of
//                    16; the last one only with the normalised read-out)
//
//   phase 1 (a_scan_kernel):  one workgroup per head, the A chain of the block form; the C x C work the S
//                             recurrence needs (c_t, Z, NQ) is done one block behind by a wave that would
//                             otherwise wait for the factorisation of the next block
//   phase 2 (s_rows_kernel):  one wave per (head, 16-row slab of S); operands come straight from
//                             global memory in MFMA operand layout, no LDS and no barriers
//           (s_rows_lds_kernel, many heads): one workgroup per head, operands shared through LDS
//
// Every kernel also takes a time segment of the sequence instead of the whole of it: the time-parallel mode
// (driver at the end of this file, boundary states in vla_segments.hip) runs the segments concurrently.
#include "vla_mfma_util.h"

#include <type_traits>

namespace vla {
namespace {

// ------------------------------------------------------------------------------------------ phase 1
// Two-wave workgroups (d <= 64) are compiled for three waves per SIMD.
//
// MAPF (time-parallel mode, d <= 64): the workgroup also forms the affine map S_end = S_start P + Q of its
// segment, which the composition of the segment-start states needs.  Rows of S are independent, so P is what the
// rows of the identity evolve into with v = 0 and Q what a zero state evolves into with the real v; both run here
// one block behind the A chain, on the operands that are still in LDS (K^ and W of the previous block in a second
// copy, Z and c from the C x C pass), instead of in a pass of their own that reads them back from the workspace.
// The 2 d/16 row slabs of 16 rows are dealt out over the waves.
template <int D, int NW, typename IO, bool MAPF = false>
__global__ void __launch_bounds__(64 * NW, (NW == 2 && !MAPF) ? 3 : 2) a_scan_kernel(ForwardArgs a) {
  static_assert(NW >= 2, "the C x C pass of the previous block runs on a second wave");
  constexpr int NKB = MAPF ? 2 : 1;            // copies of K^ and W in LDS
  constexpr int NSLAB = D / 16;                // 16-row slabs of a d x d state
  constexpr int SPW = 2 * NSLAB / NW;          // slabs of the map (Q run, then P run) per wave
  static_assert(!MAPF || NSLAB % NW == 0, "whole slabs per wave, the Q run in its first slots");
  constexpr int QSL = NSLAB / NW;              // slots i < QSL of a wave are Q-run slabs, the others P-run slabs
  constexpr int SL = D / NW;
  constexpr int NJ = SL / 16;
  constexpr int NB = D / 16;
  constexpr int LD = D + 4;
  constexpr int NT = 64 * NW;
  // Staging: a token row is split over TPR threads of EPT elements each.  For the power-of-two head sizes every
  // thread stages; at d = 96 a row takes 6 threads of 16 elements in a group of 8 (two lanes of each group and
  // the third wave stage nothing), so that a row never straddles a wave and sums with a power-of-two shuffle.
  constexpr int TPR0 = NT / C;
  constexpr bool PADDED = (TPR0 & (TPR0 - 1)) != 0;
  constexpr int EPT = PADDED ? 16 : C * D / NT;
  constexpr int TPR = PADDED ? 8 : D / EPT;
  static_assert(EPT % 4 == 0 && TPR <= 16 && (TPR & (TPR - 1)) == 0 && C * TPR <= NT && D % EPT == 0 &&
                D / EPT <= TPR, "staging layout");

  __shared__ __align__(16) float Ksb[NKB][C * LD];
  __shared__ __align__(16) float Qs[C * LD];
  __shared__ __align__(16) float Ys[C * LD];
  __shared__ __align__(16) float Wbb[NKB][D * LT];
  __shared__ __align__(16) float Gp[NW][2][C * LT];
  // MAPF: Z [t][s] and -c of the previous block live in Y^T's array, which is dead between barrier (2) of a block
  // and the first barrier of the next one: exactly the window in which they are written and read (four
  // workgroups of 40 KB share a compute unit; separate arrays would make it three)
  static_assert(C * LD >= C * LT + C, "Z and c fit the Y^T array");
  float* const Zs = Ys;
  float* const cvs = Ys + C * LT;
  // kept for one more block (two copies, by block parity): the wave that turns them into c, Z, NQ reads the
  // previous block's while the factorisation of the current block writes its own
  __shared__ __align__(16) float Lis[2][C * LT];   // L^{-1} [t][s]
  __shared__ __align__(16) float Lrs[2][C * LT];   // L [t][s]
  __shared__ __align__(16) float GQs[2][C * LT];   // GQ [s][t]
  __shared__ __align__(16) float wn2p[NW][C];

  // One workgroup per (head, time segment); with a single segment it walks the whole sequence.
  const int head = blockIdx.x / a.n_seg;
  const int seg = blockIdx.x - head * a.n_seg;
  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int c = lane & 15;
  const int g = lane >> 4;
  const int tb = seg * a.seg_blocks * C;                                   // first token of the segment
  const int T = min(a.T, tb + a.seg_blocks * C);                           // one past its last token
  const float eps = a.eps;
  const bool fmap = a.feature_map != 0;   // q and k are replaced by ELU(x) + 1 as they are staged
  const int col0 = SL * w;
  const int nblk = (a.T + C - 1) / C;                                      // blocks of the whole sequence

  float* wsh = a.ws + static_cast<size_t>(head) * head_stride(nblk, D);
  float* RN = wsh + off_rn(nblk, D);
  float* WT = wsh + off_wt(nblk, D);
  float* SMp = wsh + off_sm(nblk, D);

  f4 At[NB][NJ];
  {
    const float* A0 = a.seg_A ? a.seg_A + static_cast<size_t>(blockIdx.x) * D * D
                              : (a.A0 ? a.A0 + static_cast<size_t>(head) * D * D : nullptr);
    const float diag = 1.0f / a.lambda0;
    const int arc = (4 * g) * D + col0 + c;
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
      }
  }

  const size_t slab = static_cast<size_t>(head) * static_cast<size_t>(a.T) * D;
  const IO* qh = static_cast<const IO*>(a.q) + slab;
  const IO* kh = static_cast<const IO*>(a.k) + slab;
  const int srow = tid / TPR;
  const int sseg = (tid % TPR) * EPT;
  const bool stager = !PADDED || (tid < C * TPR && sseg < D);    // this thread holds a row segment
  const bool stage_wave = !PADDED || tid < C * TPR;              // uniform per wave

  RawRow<IO, EPT> kpre, qpre;
  auto prefetch = [&](int t0) {
    if (stager) {
      const int tr = t0 + srow;
      const unsigned koff = static_cast<unsigned>((tr < T ? tr : T - 1) * D + sseg);
      kpre.load(kh + koff);
      qpre.load(qh + koff);
    }
  };
  if (tb < T) prefetch(tb);

  int cc = c;  // opaque copy: keeps the (c == t) masks from being hoisted into 16 registers
  asm volatile("" : "+v"(cc));

  // c_t, Z = (I + strict_lower(L) diag(c))^{-1} and -NQ^T of one block from what its factorisation left in LDS
  // copy `pb`; one wave.  Results go to the block's record in the workspace.
  auto cz_pass = [&](int pb, float* smb) {
    float m[C];  // lane c: row c of L
#pragma unroll
    for (int s4 = 0; s4 < C; s4 += 4) {
      const f4 lr = lds4(&Lrs[pb][c * LT + s4]);
#pragma unroll
      for (int e = 0; e < 4; ++e) m[s4 + e] = lr[e];
    }
    const float dl = Lrs[pb][c * LT + c];  // L_cc
    float wn2 = 0.0f;
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) wn2 += wn2p[ww][c];
    // hardware reciprocal and square root (1 ulp): c_t only scales the write direction
    const float rdl = __builtin_amdgcn_rcpf(dl);
    const float an = __builtin_amdgcn_sqrtf(wn2) * rdl;                // ||A_t k^_t|| = ||w_t|| / L_tt
    const float cs = rdl * __builtin_amdgcn_rcpf(fmaxf(an, eps));      // alpha^_t = c_t w_t
    float nm[C], Zr[C];
    float ncs = -cs;
    asm volatile("s_nop 1" : "+v"(ncs));   // a DPP read of a VGPR needs 2 wait states after its write
    scale_cols<0>(m, nm, ncs);             // lane t: -L[t][s] c_s
    asm volatile("s_nop 1" : "+v"(nm[0]));
    z_rows<0>(nm, Zr, cc);
    const f4 la = lds4(&Lis[pb][c * LT + 4 * g]);
    f4 hq = f4{0, 0, 0, 0};   // H = L^{-1} GQ
#pragma unroll
    for (int r = 0; r < 4; ++r) hq = mfma16(la[r], GQs[pb][(4 * g + r) * LT + c], hq);
    f4 nq;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int sidx = 4 * g + r;
      const float csr = __shfl(cs, sidx);
      nq[r] = (sidx <= c) ? -(csr * hq[r]) : 0.0f;
    }
    if (g == 0) {
#pragma unroll
      for (int t = 0; t < C; ++t) smb[t * C + c] = Zr[t];
      smb[2 * C * C + c] = -cs;
      if constexpr (MAPF) {
#pragma unroll
        for (int t = 0; t < C; ++t) Zs[t * LT + c] = Zr[t];
        cvs[c] = -cs;
      }
    }
    *reinterpret_cast<f4*>(smb + C * C + c * C + 4 * g) = nq;  // -NQ^T[t = c][s = 4g + r]
  };

  // ---- the segment's affine map (MAPF): mst[i][b][r] = X[row0_i + c][16b + 4g + r] for this wave's slabs
  const bool do_map = MAPF && seg != a.n_seg - 1;   // nothing follows the last segment
  const IO* vh = static_cast<const IO*>(a.v) + static_cast<size_t>(head) * static_cast<size_t>(a.T) * D;
  f4 mst[MAPF ? SPW : 1][NB];
  IO vcur[MAPF ? SPW : 1][4] = {}, vnext[MAPF ? SPW : 1][4] = {};
  if constexpr (MAPF) {
#pragma unroll
    for (int i = 0; i < SPW; ++i) {
      const int sl = w + NW * i;                       // slab: Q run for sl < NSLAB, then P run
      const bool p_run = sl >= NSLAB;
      const int row0 = (sl % NSLAB) * 16;
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r = 0; r < 4; ++r) mst[i][b][r] = (p_run && row0 + c == 16 * b + 4 * g + r) ? 1.0f : 0.0f;
    }
  }
  // v of the block starting at t0 in accumulator layout, for the Q-run slabs (rows past the end: the last row)
  auto load_map_v = [&](int t0, IO (&vv)[MAPF ? SPW : 1][4]) {
    if constexpr (MAPF) {
#pragma unroll
      for (int i = 0; i < QSL; ++i) {
        const int sl = w + NW * i;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int t = t0 + 4 * g + r;
          vv[i][r] = vh[static_cast<size_t>(t < T ? t : T - 1) * D + sl * 16 + c];
        }
      }
    }
  };
  // one block of the S recurrence on this wave's slabs: operands of the block in LDS copy `kb`
  auto map_step = [&](int t0, int kb, const IO (&vv)[MAPF ? SPW : 1][4]) {
    if constexpr (MAPF) {
      const f4 za = lds4(&Zs[c * LT + 4 * g]);
      const f4 cg = lds4(&cvs[4 * g]);
#pragma unroll
      for (int i = 0; i < SPW; ++i) {
        f4 ft = f4{0, 0, 0, 0};
        if (i < QSL) {   // known at compile time: the P run starts from v = 0
          if (t0 + C <= T) {   // uniform: only the ragged last block masks rows past the end
#pragma unroll
            for (int r = 0; r < 4; ++r) ft[r] = neg_widen(vv[i][r]);
          } else {
#pragma unroll
            for (int r = 0; r < 4; ++r) ft[r] = (t0 + 4 * g + r < T) ? neg_widen(vv[i][r]) : 0.0f;
          }
        }
#pragma unroll
        for (int b = 0; b < NB; ++b) {
          const f4 ka = lds4(&Ksb[kb][c * LD + 16 * b + 4 * g]);
#pragma unroll
          for (int r = 0; r < 4; ++r) ft = mfma16(ka[r], mst[i][b][r], ft);
        }
        f4 et = f4{0, 0, 0, 0};
#pragma unroll
        for (int r = 0; r < 4; ++r) et = mfma16(za[r], ft[r], et);
        const f4 ce = et * cg;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
          const f4 wa = lds4(&Wbb[kb][(16 * b + c) * LT + 4 * g]);
#pragma unroll
          for (int r = 0; r < 4; ++r) mst[i][b] = mfma16(wa[r], ce[r], mst[i][b]);
        }
      }
    }
  };

  int blk = seg * a.seg_blocks;
  int it = 0;   // blocks done by this workgroup
  __builtin_amdgcn_s_setprio(1);
  for (int t0 = tb; t0 < T; t0 += C, ++blk, ++it) {
    const int pb = it & 1;
    float* Ks = Ksb[MAPF ? pb : 0];
    float* Wb = Wbb[MAPF ? pb : 0];
    // ---- stage K^ and Q (LDS); 1 / max(||k||, eps) per token goes to the workspace
    if (stage_wave) {
      float kx[EPT];
      const bool live = t0 + srow < T && stager;
      if (stager) {
        kpre.unpack(kx);
      } else {
#pragma unroll
        for (int e = 0; e < EPT; ++e) kx[e] = 0.0f;
      }
      if (fmap) {
#pragma unroll
        for (int e = 0; e < EPT; ++e) kx[e] = elu_plus_one(kx[e]);
      }
      const bool ragged = t0 + C > T;   // uniform: only the last block masks rows past the end
      if (ragged || PADDED) {
#pragma unroll
        for (int e = 0; e < EPT; ++e) kx[e] = live ? kx[e] : 0.0f;
      }
      float ss = 0.0f;
#pragma unroll
      for (int e = 0; e < EPT; ++e) ss = fmaf(kx[e], kx[e], ss);
#pragma unroll
      for (int off = TPR / 2; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
      // 1 / max(||k||, eps) = rsqrt(max(||k||^2, eps^2)): hardware reciprocal square root, one Newton step
      const float sm = fmaxf(ss, eps * eps);
      float rn = __builtin_amdgcn_rsqf(sm);
      rn = rn * fmaf(-0.5f * sm * rn, rn, 1.5f);
      if (stager) {
        if (sseg == 0) RN[t0 + srow] = live ? rn : 0.0f;   // rows past the end: zero keys
#pragma unroll
        for (int e = 0; e < EPT; e += 4) {
          *reinterpret_cast<f4*>(&Ks[srow * LD + sseg + e]) =
              f4{kx[e] * rn, kx[e + 1] * rn, kx[e + 2] * rn, kx[e + 3] * rn};
        }
        qpre.unpack(kx);
        if (fmap) {
#pragma unroll
          for (int e = 0; e < EPT; ++e) kx[e] = elu_plus_one(kx[e]);
        }
        if (ragged) {
#pragma unroll
          for (int e = 0; e < EPT; ++e) kx[e] = live ? kx[e] : 0.0f;
        }
#pragma unroll
        for (int e = 0; e < EPT; e += 4)
          *reinterpret_cast<f4*>(&Qs[srow * LD + sseg + e]) = f4{kx[e], kx[e + 1], kx[e + 2], kx[e + 3]};
      }
    }
    __syncthreads();  // (1)
    if (t0 + C < T) prefetch(t0 + C);
    if (do_map) load_map_v(t0, vnext);   // consumed one block later

    // ---- Y^T = K^ A0 and the partial Gram matrices
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
    {
      f4 gg = f4{0, 0, 0, 0}, gq = f4{0, 0, 0, 0};
#pragma unroll
      for (int jn = 0; jn < NJ; ++jn) {
        const int o4 = c * LD + col0 + 16 * jn + 4 * g;
        const f4 ya = lds4(&Ys[o4]);
        const f4 kb = lds4(&Ks[o4]);
        const f4 qb = lds4(&Qs[o4]);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          gg = mfma16(ya[r], kb[r], gg);
          gq = mfma16(ya[r], qb[r], gq);
        }
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        Gp[w][0][(4 * g + r) * LT + c] = gg[r];
        Gp[w][1][(4 * g + r) * LT + c] = gq[r];
      }
    }
    __syncthreads();  // (2)

    // ---- one wave: Cholesky of I + G and L^{-1} (lanes <32 rows of L, lanes >=32 columns of L^{-1});
    //      another wave meanwhile: c, Z, NQ of the previous block
    const int sw = it % NW;
    const int sw2 = (it + 1) % NW;
    if (w == sw) {
      __builtin_amdgcn_s_setprio(3);   // the dependent chain is what the other wave waits for: issue it first
      const bool lower = lane < 32;
      float m[C];
#pragma unroll
      for (int s4 = 0; s4 < C; s4 += 4) {
        f4 acc = lds4(&Gp[0][0][c * LT + s4]);
        f4 acq = lds4(&Gp[0][1][c * LT + s4]);
#pragma unroll
        for (int ww = 1; ww < NW; ++ww) {
          acc += lds4(&Gp[ww][0][c * LT + s4]);
          acq += lds4(&Gp[ww][1][c * LT + s4]);
        }
        if (g == 1) *reinterpret_cast<f4*>(&GQs[pb][c * LT + s4]) = acq;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          m[s4 + e] = (lower ? acc[e] : 0.0f) + ((s4 + e) == cc ? 1.0f : 0.0f);
      }
#pragma unroll
      for (int t = 0; t < C; ++t) {
        const float p = readlane(m[t], t);
        const float ri = __builtin_amdgcn_rsqf(p);  // 1 ulp; L only has to satisfy L L^T = I + G to rounding
        const float li = m[t] * ri;
        m[t] = li;
#pragma unroll
        for (int j = t + 1; j < C; ++j) m[j] = fmaf(-li, readlane(li, j), m[j]);
      }
      if (g == 0) {  // rows of L
#pragma unroll
        for (int s4 = 0; s4 < C; s4 += 4)
          *reinterpret_cast<f4*>(&Lrs[pb][c * LT + s4]) = f4{m[s4], m[s4 + 1], m[s4 + 2], m[s4 + 3]};
      }
      if (g == 2) {  // columns of L^{-1}
#pragma unroll
        for (int t = 0; t < C; ++t) Lis[pb][t * LT + c] = m[t];
      }
      __builtin_amdgcn_s_setprio(1);
    } else if (w == sw2 && it > 0) {
      __builtin_amdgcn_s_setprio(3);
      cz_pass(pb ^ 1, SMp + static_cast<size_t>(blk - 1) * SMB);
      __builtin_amdgcn_s_setprio(1);
    }
    __syncthreads();  // (3)

    // ---- W^T = L^{-1} Y^T -> LDS and workspace; partial norms
    const f4 la = lds4(&Lis[pb][c * LT + 4 * g]);
    f4 nwt[NJ];
    {
      f4 n2 = f4{0, 0, 0, 0};
      float* wg = WT + static_cast<size_t>(blk) * D * C;
#pragma unroll
      for (int jn = 0; jn < NJ; ++jn) {
        f4 acc = f4{0, 0, 0, 0};
#pragma unroll
        for (int r = 0; r < 4; ++r) acc = mfma16(la[r], yt[jn][r], acc);
        nwt[jn] = -acc;
        n2 += acc * acc;
        *reinterpret_cast<f4*>(&Wb[(col0 + 16 * jn + c) * LT + 4 * g]) = acc;
        *reinterpret_cast<f4*>(wg + (col0 + 16 * jn + c) * C + 4 * g) = acc;
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) n2[r] = row_sum16(n2[r]);
      if (c == 0) *reinterpret_cast<f4*>(&wn2p[w][4 * g]) = n2;
    }
    // ---- the map, one block behind: Z and c of block it - 1 were formed before barrier (3), its K^ and W sit in
    //      the other LDS copy, which is not written again before barrier (4)
    if constexpr (MAPF) {
      if (do_map) {
        __builtin_amdgcn_s_setprio(0);   // off the A chain's path: behind the other workgroups' work
        if (it > 0) map_step(t0 - C, pb ^ 1, vcur);
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int i = 0; i < QSL; ++i)
#pragma unroll
          for (int r = 0; r < 4; ++r) vcur[i][r] = vnext[i][r];
      }
    }
    __syncthreads();  // (4)

    // ---- A -= W W^T
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const f4 wa = lds4(&Wb[(16 * b + c) * LT + 4 * g]);
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int jn = 0; jn < NJ; ++jn) At[b][jn] = mfma16(wa[r], nwt[jn][r], At[b][jn]);
    }
  }
  // c, Z, NQ of the last block: everything it needs was written before the last barrier
  if (it > 0 && w == it % NW) cz_pass((it - 1) & 1, SMp + static_cast<size_t>(blk - 1) * SMB);
  if constexpr (MAPF) {
    if (do_map && it > 0) {   // uniform over the workgroup
      __syncthreads();        // Z and c of the last block
      map_step((blk - 1) * C, (it - 1) & 1, vcur);
#pragma unroll
      for (int i = 0; i < SPW; ++i) {
        const int sl = w + NW * i;
        float* out = a.seg_PQ + (static_cast<size_t>(blockIdx.x) * 2 + (sl >= NSLAB ? 0 : 1)) * D * D;
        const int row0 = (sl % NSLAB) * 16;
#pragma unroll
        for (int b = 0; b < NB; ++b)
          *reinterpret_cast<f4*>(out + (row0 + c) * D + 16 * b + 4 * g) = mst[i][b];
      }
    }
  }

  if (a.A_T && seg == a.n_seg - 1) {
    float* AT = a.A_T + static_cast<size_t>(head) * D * D;
    int g2 = g, c2 = c;
    asm volatile("" : "+v"(g2), "+v"(c2));
    const int arc = (4 * g2) * D + col0 + c2;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int jn = 0; jn < NJ; ++jn)
#pragma unroll
        for (int r = 0; r < 4; ++r) AT[arc + (16 * b + r) * D + 16 * jn] = At[b][jn][r];
  }
}

// ------------------------------------------------------------------------------------------ phase 2
// One wave per (head, time segment, 16-row slab of S), no LDS and no barriers: the most waves when heads are
// few.  st[b][r] = S[row0 + c][16b + 4g + r]; the operands of a block (W, Z, -NQ^T, -c from the workspace, the raw
// k and q, and 1 / ||k|| per token, from which k^ is re-formed) come straight from global memory in MFMA operand
// layout.
//
// MAP = false: the recurrence proper: reads q, writes o.
// MAP = true:  the affine map S_end = S_start P + Q of one segment, for the time-parallel mode.  Rows of S
//              are independent, so row i of P is what row i of the identity evolves into with v = 0, and Q is
//              what a zero state evolves into with the real v: twice the slabs per (head, segment),
//              nothing read from q and nothing written to o; the end states go to seg_PQ.
//
// Workgroup ids are dealt round-robin over the 8 XCDs, each with its own L2; the id is decoded so that all
// waves of one (head, segment) sit on the same XCD and share the operands they all read through its L2.
template <int D, int DEPTH, typename IO, bool MAP>
__global__ void __launch_bounds__(64) s_rows_kernel(ForwardArgs a) {
  constexpr int NB = D / 16;
  constexpr int NSLAB = D / 16;
  constexpr int WPH = MAP ? 2 * NSLAB : NSLAB;       // waves per (head, segment)
  const int xcd = blockIdx.x & 7;
  const int rest = blockIdx.x >> 3;
  const int hs = (rest / WPH) * 8 + xcd;             // head * n_seg + seg
  const int grp = rest % WPH;
  if (hs >= a.n_heads * a.n_seg) return;
  const int head = hs / a.n_seg;
  const int seg = hs - head * a.n_seg;
  const bool p_run = MAP && grp >= NSLAB;            // identity rows, v = 0
  const int row0 = (grp % NSLAB) * 16;
  const int lane = threadIdx.x;
  const int c = lane & 15;
  const int g = lane >> 4;
  const int nblk = (a.T + C - 1) / C;
  const int bb = seg * a.seg_blocks;                 // block range of the segment
  const int be = min(nblk, bb + a.seg_blocks);
  const int T = min(a.T, be * C);
  if (MAP && seg == a.n_seg - 1) return;             // nothing follows the last segment

  const float* wsh = a.ws + static_cast<size_t>(head) * head_stride(nblk, D);
  const float* RN = wsh + off_rn(nblk, D);
  const float* WT = wsh + off_wt(nblk, D);
  const float* SMp = wsh + off_sm(nblk, D);
  const size_t slab = static_cast<size_t>(head) * static_cast<size_t>(a.T) * D;
  const IO* qh = static_cast<const IO*>(a.q) + slab;
  const IO* kh = static_cast<const IO*>(a.k) + slab;
  const bool fmap = a.feature_map != 0;   // q and k are replaced by ELU(x) + 1 as they are consumed
  const bool norm_out = a.normalise_output != 0;   // o_t is divided by max(q_t . zkey_t, eps)
  const IO* vh = static_cast<const IO*>(a.v) + slab;
  IO* oh = static_cast<IO*>(a.o) + slab;

  f4 st[NB];
  if constexpr (MAP) {
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int r = 0; r < 4; ++r) st[b][r] = (p_run && row0 + c == 16 * b + 4 * g + r) ? 1.0f : 0.0f;
  } else {
    const float* S0 = a.seg_S ? a.seg_S + static_cast<size_t>(hs) * D * D
                              : (a.S0 ? a.S0 + static_cast<size_t>(head) * D * D : nullptr);
#pragma unroll
    for (int b = 0; b < NB; ++b)
      st[b] = S0 ? *reinterpret_cast<const f4*>(S0 + (row0 + c) * D + 16 * b + 4 * g) : f4{0, 0, 0, 0};
  }

  // operands of one block, in MFMA operand layout, straight from global memory
  struct Ops {
    f4 wa[NB];
    RawRow<IO, 4> ka[NB], qa[NB];
    float rn;           // 1 / max(||k||, eps) of token row c (0 past the end)
    f4 za, nqa, ncg;
    f4 rd;              // 1 / max(q_t . zkey_t, eps) for t = 4g + r (normalised read-out only)
    IO v[4];
  };
  // Addresses are a per-block uniform base (scalar registers) plus lane-constant 32-bit offsets, so that a
  // load costs no vector address arithmetic; only the ragged last block clamps its token rows.
  const unsigned wo = static_cast<unsigned>(c * C + 4 * g);   // W row c of a 16-column slice; Z / NQ row c
  const unsigned vo = static_cast<unsigned>(4 * g * D + row0 + c);  // v and o: token 4g, column row0 + c
  auto load_ops = [&](int blk, Ops& o) {
    const IO* kb = kh + static_cast<size_t>(blk) * (C * D);
    const float* wb = WT + static_cast<size_t>(blk) * (D * C);
    const float* sp = SMp + static_cast<size_t>(blk) * SMB;
    const IO* qb = qh + static_cast<size_t>(blk) * (C * D);
    const IO* vb = vh + static_cast<size_t>(blk) * (C * D);
    const int lim = T - 1 - blk * C;                          // last live token row of this block
    const unsigned qo = static_cast<unsigned>(min(c, lim) * D + 4 * g);   // rows past the end: a copy of the last
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      o.ka[b].load(kb + qo + 16 * b);
      o.wa[b] = *reinterpret_cast<const f4*>(wb + wo + 16 * b * C);
      if constexpr (!MAP) o.qa[b].load(qb + qo + 16 * b);
    }
    o.rn = RN[blk * C + c];
    o.za = *reinterpret_cast<const f4*>(sp + wo);
    if constexpr (!MAP) o.nqa = *reinterpret_cast<const f4*>(sp + C * C + wo);
    o.ncg = *reinterpret_cast<const f4*>(sp + 2 * C * C + 4 * g);
    if constexpr (!MAP) {
      if (norm_out) o.rd = *reinterpret_cast<const f4*>(sp + 2 * C * C + C + 4 * g);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r)
      o.v[r] = vb[static_cast<unsigned>(min(4 * g + r, lim) * D + row0 + c)];
  };

  auto compute = [&](int blk, const Ops& cur) {
    const int t0 = blk * C;
    IO* ob = oh + static_cast<size_t>(blk) * (C * D);
    // Rows of q past the end hold a copy of the last token (clamped loads); row t of the read-out depends on
    // row t of q only, and those rows are never stored, so they need no masking.
    f4 ft, ot = f4{0, 0, 0, 0};
#pragma unroll
    for (int r = 0; r < 4; ++r) ft[r] = (!p_run && t0 + 4 * g + r < T) ? -widen(cur.v[r]) : 0.0f;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      float kx[4], qx[4];
      cur.ka[b].unpack(kx);
      if (fmap) {
#pragma unroll
        for (int r = 0; r < 4; ++r) kx[r] = elu_plus_one(kx[r]);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) kx[r] *= cur.rn;   // the same product the A scan formed k^ with
      if constexpr (!MAP) {
        cur.qa[b].unpack(qx);
        if (fmap) {
#pragma unroll
          for (int r = 0; r < 4; ++r) qx[r] = elu_plus_one(qx[r]);
        }
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        ft = mfma16(kx[r], st[b][r], ft);
        if constexpr (!MAP) ot = mfma16(qx[r], st[b][r], ot);
      }
    }
    f4 et = f4{0, 0, 0, 0};
#pragma unroll
    for (int r = 0; r < 4; ++r) et = mfma16(cur.za[r], ft[r], et);
    if constexpr (!MAP) {
#pragma unroll
      for (int r = 0; r < 4; ++r) ot = mfma16(cur.nqa[r], et[r], ot);
      if (norm_out) ot *= cur.rd;
      if (t0 + C <= T) {   // uniform: only the ragged last block predicates its stores
        io_store2(ob + vo, ob + vo + D, ot[0], ot[1]);
        io_store2(ob + vo + 2 * D, ob + vo + 3 * D, ot[2], ot[3]);
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if (t0 + 4 * g + r < T) io_store(ob + vo + r * D, ot[r]);
        }
      }
    }
    const f4 ce = et * cur.ncg;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int r = 0; r < 4; ++r) st[b] = mfma16(cur.wa[b][r], ce[r], st[b]);
  };

  // Operands are fetched DEPTH blocks ahead into rotating register sets (the loop is unrolled by DEPTH + 1
  // to keep them static).
  if constexpr (DEPTH == 2) {
    Ops o0, o1, o2;
    if (bb < be) load_ops(bb, o0);
    if (bb + 1 < be) load_ops(bb + 1, o1);
    for (int blk = bb; blk < be; blk += 3) {
      if (blk + 2 < be) load_ops(blk + 2, o2);
      compute(blk, o0);
      if (blk + 3 < be) load_ops(blk + 3, o0);
      if (blk + 1 < be) compute(blk + 1, o1);
      if (blk + 4 < be) load_ops(blk + 4, o1);
      if (blk + 2 < be) compute(blk + 2, o2);
    }
  } else {
    Ops o0, o1;
    if (bb < be) load_ops(bb, o0);
    for (int blk = bb; blk < be; blk += 2) {
      if (blk + 1 < be) load_ops(blk + 1, o1);
      compute(blk, o0);
      if (blk + 2 < be) load_ops(blk + 2, o0);
      if (blk + 1 < be) compute(blk + 1, o1);
    }
  }

  float* out = nullptr;
  if constexpr (MAP) {
    out = a.seg_PQ + (static_cast<size_t>(hs) * 2 + (p_run ? 0 : 1)) * D * D;
  } else if (a.S_T && seg == a.n_seg - 1) {
    out = a.S_T + static_cast<size_t>(head) * D * D;
  }
  if (out) {
#pragma unroll
    for (int b = 0; b < NB; ++b)
      *reinterpret_cast<f4*>(out + (row0 + c) * D + 16 * b + 4 * g) = st[b];
  }
}

template <int D, typename IO, bool MAP>
hipError_t launch_s_rows(const ForwardArgs& a, hipStream_t stream) {
  ForwardArgs args = a;
  void* params[] = {&args};
  constexpr int kDepth = D <= 64 ? 2 : 1;  // register budget: three operand sets only fit up to d = 64
  constexpr int kWph = (MAP ? 2 : 1) * (D / 16);
  const long long hs = static_cast<long long>(a.n_heads) * a.n_seg;
  const long long wgs = (hs + 7) / 8 * 8 * kWph;
  if (wgs > 0x7fffffffLL) return hipErrorInvalidValue;
  const unsigned grid = static_cast<unsigned>(wgs);
  return hipLaunchKernel(reinterpret_cast<const void*>(&s_rows_kernel<D, kDepth, IO, MAP>), dim3(grid),
                         dim3(64), params, 0, stream);
}

// ------------------------------------------------------------------------------- phase 2, shared operands
// The same recurrence with one workgroup per (head, time segment): one wave per 16-row slab of S (twice as
// many waves for the map pass: Q-run slabs, then P-run slabs), the block's operands fetched once for all of
// them and handed round through LDS.  Used when there are enough (head, segment) pairs to fill the chip: the
// per-wave kernel above then reads the same operands d/16 times over and every wave waits on its own stream.
//
// Pipeline, one barrier per block: the data of block n is requested in iteration n - 3 (two register sets),
// written to LDS stage n % 2 in iteration n - 1 (after that iteration's barrier, which every wave reaches only
// when it is done reading the stage for block n - 2) and consumed in iteration n.  Registers are capped at 128
// so that four workgroups (d <= 64) share a compute unit and 1024 (head, segment) pairs run in one round.
//
// RECT: value heads of another size than the key heads (S has a.d_v rows, D columns).  The workgroup keeps its
// D / 16 waves per run (they stage the operands, whose size follows D) and the d_v / 16 row slabs of S go to
// them in turn: slab t to wave t % (D / 16), NJV = slots per wave; a wave with no slab in a slot skips it.
// The P run always has D / 16 slabs, one per wave.
template <int D, int NJV, bool RECT, typename IO, bool MAP>
__global__ void __launch_bounds__(64 * (D / 16) * (MAP ? 2 : 1), NJV == 1 ? 4 : 2) s_rows_lds_kernel(ForwardArgs a) {
  static_assert(RECT || NJV == 1, "square heads: one slab per wave");
  constexpr int NB = D / 16;
  constexpr int NSLAB = D / 16;                  // waves of a run
  constexpr int NT = 64 * NSLAB * (MAP ? 2 : 1);
  constexpr int LD = D + 4;
  constexpr int CH = 4 * D;                     // 16-byte pieces of K^ (and of W, and 4-element pieces of q)
  static_assert(NT == (MAP ? 2 * CH : CH), "one piece of each big operand per thread");
  constexpr int NST = 2;
  struct Stage {
    float Ks[C * LD];      // K^ [t][j]
    float Qs[C * LD];      // q  [t][j] widened (unused by the map pass)
    float Wb[D * LT];      // W  [j][t]
    float Zs[C * LT];      // Z  [t][s]
    float NQs[C * LT];     // -NQ^T [t][s]
    float cv[2 * C];       // -c_t, then 1 / max(q_t . zkey_t, eps) (normalised read-out only)
  };
  __shared__ __align__(16) Stage stg[NST];

  const int hs = blockIdx.x;                     // head * n_seg + seg
  const int head = hs / a.n_seg;
  const int seg = hs - head * a.n_seg;
  if (MAP && seg == a.n_seg - 1) return;         // nothing follows the last segment
  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int c = lane & 15;
  const int g = lane >> 4;
  const bool p_run = MAP && w >= NSLAB;          // identity rows, v = 0
  const int DV = RECT ? a.d_v : D;               // rows of S
  const int wq = w % NSLAB;
  // slot jn of this wave: rows row_of(jn) .. + 15 of S (of the identity in the P run, which has D rows)
  auto row_of = [&](int jn) { return 16 * (wq + NSLAB * jn); };
  auto owns = [&](int jn) { return jn == 0 ? (p_run || 16 * wq < DV) : (!p_run && row_of(jn) < DV); };
  const int nblk = (a.T + C - 1) / C;
  const int bb = seg * a.seg_blocks;
  const int be = min(nblk, bb + a.seg_blocks);
  const int T = min(a.T, be * C);

  const float* wsh = a.ws + static_cast<size_t>(head) * head_stride(nblk, D);
  const float* RN = wsh + off_rn(nblk, D);
  const float* WT = wsh + off_wt(nblk, D);
  const float* SMp = wsh + off_sm(nblk, D);
  const size_t slab = static_cast<size_t>(head) * static_cast<size_t>(a.T) * D;
  const IO* qh = static_cast<const IO*>(a.q) + slab;
  const IO* kh = static_cast<const IO*>(a.k) + slab;
  const bool fmap = a.feature_map != 0;   // q and k are replaced by ELU(x) + 1 as they are consumed
  const bool norm_out = a.normalise_output != 0;   // o_t is divided by max(q_t . zkey_t, eps)
  const size_t vslab = static_cast<size_t>(head) * static_cast<size_t>(a.T) * DV;
  const IO* vh = static_cast<const IO*>(a.v) + vslab;
  IO* oh = static_cast<IO*>(a.o) + vslab;
  const size_t ssz = static_cast<size_t>(DV) * D;   // floats of S (and of Q)

  f4 st[NJV][NB];   // st[jn][b][r] = S[row_of(jn) + c][16b + 4g + r]
  if constexpr (MAP) {
#pragma unroll
    for (int jn = 0; jn < NJV; ++jn)
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          st[jn][b][r] = (p_run && jn == 0 && 16 * wq + c == 16 * b + 4 * g + r) ? 1.0f : 0.0f;
  } else {
    const float* S0 = a.seg_S ? a.seg_S + static_cast<size_t>(hs) * ssz
                              : (a.S0 ? a.S0 + static_cast<size_t>(head) * ssz : nullptr);
#pragma unroll
    for (int jn = 0; jn < NJV; ++jn)
#pragma unroll
      for (int b = 0; b < NB; ++b)
        st[jn][b] = (S0 && owns(jn)) ? *reinterpret_cast<const f4*>(S0 + (row_of(jn) + c) * D + 16 * b + 4 * g)
                                     : f4{0, 0, 0, 0};
  }

  // ---- this thread's share of a block's operands
  // big operands: piece `pc` of k and of q (row pc / (D/4), columns 4 (pc % (D/4)) ..) and of W (row
  // pc / 4 of [D][16], columns 4 (pc % 4) ..); in the map pass the first half of the threads carries K^ and
  // the second half W.  small operands: the record Z | -NQ^T | -c | denominators is 136 pieces in a row, piece
  // t on thread t (Z on 0-63, -NQ^T on 64-127 outside the map pass, -c and the denominators on 128-135); with
  // only 128 threads (d = 32 outside the map pass) the last pieces ride in a register of their own on threads 0-7.
  const int pc = MAP ? tid % CH : tid;
  const bool do_k = !MAP || tid < CH;
  const bool do_w = !MAP || tid >= CH;
  const int krow = pc / (D / 4), kcol = 4 * (pc % (D / 4));
  const int wrow = pc / 4, wcol = 4 * (pc % 4);
  constexpr bool kSepC = NT < 136;
  const int nc = (!MAP && norm_out) ? 8 : 4;   // -c (and the read-out denominators behind it)
  const bool do_sm = tid < (MAP ? 64 : 128) || (!kSepC && tid >= 128 && tid < 128 + nc);
  const bool do_c = kSepC && tid < nc;
  struct Regs {
    f4 wx, sx, cx;
    RawRow<IO, 4> kx, qx;
    float krn;          // 1 / max(||k||, eps) of token row krow (0 past the end)
    IO v[NJV][4];
  };
  // Byte offsets inside a block's records are per-thread constants (32 bits); the block's base addresses are
  // uniform (scalar registers).  Only the ragged last block has to clamp its token rows (rows past the end read
  // the last row).
  // (krow D + kcol = wrow C + wcol = 4 pc and sm_src = 4 tid: piece pc of a row-major array of 4-element pieces.)
  constexpr unsigned ES = sizeof(IO);
  static_assert(C == 16, "piece arithmetic");
  const unsigned p16 = 16u * static_cast<unsigned>(pc);      // byte offset of float piece pc
  const unsigned t16 = 16u * static_cast<unsigned>(tid);
  const unsigned kq_off = p16 * ES / 4u;                       // 4 pc elements of IO
  const unsigned w_off = p16;
  const unsigned sm_off = t16;
  const unsigned c_off = static_cast<unsigned>(2 * C * C) * 4u + t16;
  const unsigned rn_off = static_cast<unsigned>(krow) * 4u;
  unsigned v_off[NJV];   // token row 4 g, column row_of(jn) + c of a block of v (and of o)
#pragma unroll
  for (int jn = 0; jn < NJV; ++jn) v_off[jn] = static_cast<unsigned>(4 * g * DV + row_of(jn) + c) * ES;
  const bool reads_v = !p_run;   // the P run starts from v = 0 (and its rows need not exist in v)
  auto at = [](const void* base, unsigned byte_off) { return static_cast<const char*>(base) + byte_off; };
  auto fetch = [&](int blk, Regs& r) {
    const size_t tok = static_cast<size_t>(blk) * (C * D);
    const IO* kb = kh + tok;
    const IO* qb = qh + tok;
    const IO* vb = vh + static_cast<size_t>(blk) * (C * DV);
    const float* wb = WT + tok;
    const float* sb = SMp + static_cast<size_t>(blk) * SMB;
    const float* rb = RN + static_cast<size_t>(blk) * C;
    const int lim = T - 1 - blk * C;   // last live token row of the block
    unsigned kq = kq_off, vo[NJV][4];
#pragma unroll
    for (int jn = 0; jn < NJV; ++jn)
#pragma unroll
      for (int i = 0; i < 4; ++i) vo[jn][i] = v_off[jn] + static_cast<unsigned>(i * DV) * ES;
    if (lim < C - 1) {   // uniform
      kq = static_cast<unsigned>(min(krow, lim) * D + kcol) * ES;
#pragma unroll
      for (int jn = 0; jn < NJV; ++jn)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          vo[jn][i] = static_cast<unsigned>(min(4 * g + i, lim) * DV + row_of(jn) + c) * ES;
    }
    if (do_w) r.wx = *reinterpret_cast<const f4*>(at(wb, w_off));
    if (do_sm) r.sx = *reinterpret_cast<const f4*>(at(sb, sm_off));
    if constexpr (kSepC) {
      if (do_c) r.cx = *reinterpret_cast<const f4*>(at(sb, c_off));
    }
    if (do_k) {
      r.kx.load(reinterpret_cast<const IO*>(at(kb, kq)));
      r.krn = *reinterpret_cast<const float*>(at(rb, rn_off));
    }
    if constexpr (!MAP) r.qx.load(reinterpret_cast<const IO*>(at(qb, kq)));
#pragma unroll
    for (int jn = 0; jn < NJV; ++jn) {
      if (RECT ? (reads_v && owns(jn)) : true) {
#pragma unroll
        for (int i = 0; i < 4; ++i) r.v[jn][i] = *reinterpret_cast<const IO*>(at(vb, vo[jn][i]));
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) r.v[jn][i] = IO{};
      }
    }
  };
  auto put = [&](const Regs& r, Stage& s) {
    if (do_k) {   // k^ = k / max(||k||, eps): the same product the A scan formed it with
      float x[4];
      r.kx.unpack(x);
      if (fmap) {
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] = elu_plus_one(x[i]);
      }
      *reinterpret_cast<f4*>(&s.Ks[krow * LD + kcol]) = f4{x[0] * r.krn, x[1] * r.krn, x[2] * r.krn, x[3] * r.krn};
    }
    if (do_w) *reinterpret_cast<f4*>(&s.Wb[wrow * LT + wcol]) = r.wx;
    if (do_sm) {
      // Z and -NQ^T rows are 16 floats in the workspace and LT in LDS
      if (tid < 64) *reinterpret_cast<f4*>(&s.Zs[(tid / 4) * LT + 4 * (tid % 4)]) = r.sx;
      else if (tid < 128) *reinterpret_cast<f4*>(&s.NQs[((tid - 64) / 4) * LT + 4 * (tid % 4)]) = r.sx;
      else *reinterpret_cast<f4*>(&s.cv[4 * (tid - 128)]) = r.sx;
    }
    if constexpr (kSepC) {
      if (do_c) *reinterpret_cast<f4*>(&s.cv[4 * tid]) = r.cx;
    }
    if constexpr (!MAP) {
      float x[4];
      r.qx.unpack(x);
      if (fmap) {
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] = elu_plus_one(x[i]);
      }
      *reinterpret_cast<f4*>(&s.Qs[krow * LD + kcol]) = f4{x[0], x[1], x[2], x[3]};
    }
  };
  auto compute = [&](int blk, const Stage& s, const IO (&vv)[NJV][4]) {
    const int t0 = blk * C;
#pragma unroll
    for (int jn = 0; jn < NJV; ++jn) {
      if (RECT && !owns(jn)) continue;   // uniform over the wave
      f4 ft, ot = f4{0, 0, 0, 0};
#pragma unroll
      for (int r = 0; r < 4; ++r) ft[r] = (!p_run && t0 + 4 * g + r < T) ? -widen(vv[jn][r]) : 0.0f;
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const f4 ka = lds4(&s.Ks[c * LD + 16 * b + 4 * g]);
        f4 qa;
        if constexpr (!MAP) qa = lds4(&s.Qs[c * LD + 16 * b + 4 * g]);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          ft = mfma16(ka[r], st[jn][b][r], ft);
          if constexpr (!MAP) ot = mfma16(qa[r], st[jn][b][r], ot);
        }
      }
      const f4 za = lds4(&s.Zs[c * LT + 4 * g]);
      f4 et = f4{0, 0, 0, 0};
#pragma unroll
      for (int r = 0; r < 4; ++r) et = mfma16(za[r], ft[r], et);
      if constexpr (!MAP) {
        const f4 nqa = lds4(&s.NQs[c * LT + 4 * g]);
#pragma unroll
        for (int r = 0; r < 4; ++r) ot = mfma16(nqa[r], et[r], ot);
        if (norm_out) ot *= lds4(&s.cv[C + 4 * g]);
        // uniform block base + this lane's 32-bit byte offset (the one its v loads use)
        IO* ob = reinterpret_cast<IO*>(reinterpret_cast<char*>(oh + static_cast<size_t>(blk) * (C * DV)) + v_off[jn]);
        if (t0 + C <= T) {   // uniform: only the ragged last block predicates its stores
          io_store2(ob, ob + DV, ot[0], ot[1]);
          io_store2(ob + 2 * DV, ob + 3 * DV, ot[2], ot[3]);
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            if (t0 + 4 * g + r < T) io_store(ob + r * DV, ot[r]);
          }
        }
      }
      const f4 ce = et * lds4(&s.cv[4 * g]);
#pragma unroll
      for (int b = 0; b < NB; ++b) {
        const f4 wa = lds4(&s.Wb[(16 * b + c) * LT + 4 * g]);
#pragma unroll
        for (int r = 0; r < 4; ++r) st[jn][b] = mfma16(wa[r], ce[r], st[jn][b]);
      }
    }
  };

  // prologue: block bb into stage 0 (visible after the first barrier), bb+1 and bb+2 in flight
  Regs r0, r1;
  if (bb < be) {
    fetch(bb, r0);
    put(r0, stg[0]);
  }
  auto copy_v = [](IO (&dst)[NJV][4], const IO (&src)[NJV][4]) {
#pragma unroll
    for (int jn = 0; jn < NJV; ++jn)
#pragma unroll
      for (int i = 0; i < 4; ++i) dst[jn][i] = src[jn][i];
  };
  IO vcur[NJV][4];
  copy_v(vcur, r0.v);
  if (bb + 1 < be) fetch(bb + 1, r0);
  if (bb + 2 < be) fetch(bb + 2, r1);
  // iteration n (block bb + n): r0 holds block n+1, r1 block n+2 when n is even, the other way round when odd
  for (int n = 0; bb + n < be; n += 2) {
    {
      const int blk = bb + n;
      __syncthreads();
      IO vnext[NJV][4];
      copy_v(vnext, r0.v);
      if (blk + 1 < be) put(r0, stg[(n + 1) % NST]);
      if (blk + 3 < be) fetch(blk + 3, r0);
      compute(blk, stg[n % NST], vcur);
      copy_v(vcur, vnext);
    }
    if (bb + n + 1 < be) {
      const int blk = bb + n + 1;
      __syncthreads();
      IO vnext[NJV][4];
      copy_v(vnext, r1.v);
      if (blk + 1 < be) put(r1, stg[(n + 2) % NST]);
      if (blk + 3 < be) fetch(blk + 3, r1);
      compute(blk, stg[(n + 1) % NST], vcur);
      copy_v(vcur, vnext);
    }
  }

  float* out = nullptr;
  if constexpr (MAP) {   // per (head, segment): P [D][D], then Q [DV][D]
    out = a.seg_PQ + static_cast<size_t>(hs) * (static_cast<size_t>(D) * D + ssz) + (p_run ? 0 : D * D);
  } else if (a.S_T && seg == a.n_seg - 1) {
    out = a.S_T + static_cast<size_t>(head) * ssz;
  }
  if (out) {
#pragma unroll
    for (int jn = 0; jn < NJV; ++jn) {
      if (RECT && !owns(jn)) continue;
#pragma unroll
      for (int b = 0; b < NB; ++b)
        *reinterpret_cast<f4*>(out + (row_of(jn) + c) * D + 16 * b + 4 * g) = st[jn][b];
    }
  }
}

template <int D, int NJV, bool RECT, typename IO, bool MAP>
hipError_t launch_s_rows_lds_n(const ForwardArgs& a, hipStream_t stream) {
  ForwardArgs args = a;
  void* params[] = {&args};
  return hipLaunchKernel(reinterpret_cast<const void*>(&s_rows_lds_kernel<D, NJV, RECT, IO, MAP>),
                         dim3(a.n_heads * a.n_seg), dim3(64 * (D / 16) * (MAP ? 2 : 1)), params, 0, stream);
}
// Square heads, or (a.d_v != D) value heads of another size: slots per wave = ceil((d_v / 16) / (D / 16)).
template <int D, typename IO, bool MAP>
hipError_t launch_s_rows_lds(const ForwardArgs& a, hipStream_t stream) {
  const int dv = a.d_v > 0 ? a.d_v : D;
  if (dv == D) return launch_s_rows_lds_n<D, 1, false, IO, MAP>(a, stream);
  if (dv % 16 != 0 || dv < 16) return hipErrorInvalidValue;
  constexpr int NW = D / 16;
  constexpr int kMaxSlots = (128 / 16 + NW - 1) / NW;   // value heads up to 128
  const int slots = (dv / 16 + NW - 1) / NW;
  if (slots == 1) return launch_s_rows_lds_n<D, 1, true, IO, MAP>(a, stream);
  if constexpr (kMaxSlots >= 2) {
    if (slots == 2) return launch_s_rows_lds_n<D, 2, true, IO, MAP>(a, stream);
  }
  if constexpr (kMaxSlots >= 3) {
    if (slots == 3) return launch_s_rows_lds_n<D, 3, true, IO, MAP>(a, stream);
  }
  if constexpr (kMaxSlots >= 4) {
    if (slots == 4) return launch_s_rows_lds_n<D, 4, true, IO, MAP>(a, stream);
  }
  return hipErrorInvalidValue;
}

// true when the call switches on a separate penalty direction or the normalised read-out (the feature map
// alone runs on the plain kernels)
bool runs_on_option_kernel(const ForwardArgs& a) {
  return a.u != nullptr || a.normalise_output != 0 || a.zkey0 != nullptr || a.zkey_T != nullptr;
}

// Phase 1 and 2 over every (head, segment) of `a`.
template <int D, int NW, typename IO>
hipError_t launch_phases(const ForwardArgs& a, hipStream_t stream) {
  ForwardArgs args = a;
  void* params[] = {&args};
  const long long hs = static_cast<long long>(a.n_heads) * a.n_seg;
  if (hs * (D / 8) > 0x7fffffffLL) return hipErrorInvalidValue;   // the largest grid below: 2 D/16 waves per pair
  // A separate penalty direction or the normalised read-out: the A chain of the block kernel that carries
  // them; its records have the layout the S-row kernels below read.
  const bool general = runs_on_option_kernel(a);
  // Up to d = 64 the plain A scan also forms the per-segment affine maps of S (its registers hold them beside A).
  constexpr bool kFusedMap = D <= 64;
  // Worth it once the (head, segment) pairs fill the chip (measured at 16 heads, d = 64: 3 % faster at 1024
  // pairs, 5 % slower at 512 and below, where a block's latency counts and the maps lengthen it).
  const bool rect = a.d_v > 0 && a.d_v != D;   // value heads of another size: the A scan is the same, S has d_v rows
  const bool fused_map = kFusedMap && !general && !rect && a.n_seg > 1 && hs >= 768;
  const void* scan_fn = reinterpret_cast<const void*>(&a_scan_kernel<D, NW, IO, false>);
  if constexpr (kFusedMap) {
    if (fused_map) scan_fn = reinterpret_cast<const void*>(&a_scan_kernel<D, NW, IO, true>);
  }
  hipError_t err = general ? launch_a_scan_general(a, D, std::is_same<IO, uint16_t>::value ? 1 : 0, stream)
                           : hipLaunchKernel(scan_fn, dim3(static_cast<unsigned>(hs)), dim3(64 * NW), params, 0,
                                             stream);
  if (err != hipSuccess) return err;
  // From half a chip of (head, segment) pairs the block operands are shared through LDS by a workgroup per
  // pair; with fewer, one wave per slab of S and deep register prefetch (measured, whole call, LDS kernel
  // against the other: 240 to 255 pairs -7 to -13 % at d = 64, -8 to -25 % at d = 128; 128 pairs -3.5 and
  // -0.4 %; 9 to 32 pairs +2 to +8 %).
  // (value heads of another size: the LDS kernel at any count)
  const bool shared = rect || hs >= 128;
  auto rows = [&](auto map_tag) -> hipError_t {
    constexpr bool kMap = decltype(map_tag)::value;
    return shared ? launch_s_rows_lds<D, IO, kMap>(a, stream) : launch_s_rows<D, IO, kMap>(a, stream);
  };
  if (a.n_seg > 1) {
    // the state of S at the segment boundaries: per-segment affine maps, then their composition
    if (!fused_map) {
      err = rows(std::true_type{});
      if (err != hipSuccess) return err;
    }
    err = launch_combine(a, D, const_cast<float*>(a.seg_S), stream);
    if (err != hipSuccess) return err;
  }
  return rows(std::false_type{});
}

}  // namespace

size_t two_phase_workspace_bytes(int n_heads, int T, int d) {
  const int nblk = (T + C - 1) / C;
  return static_cast<size_t>(n_heads) * head_stride(nblk, d) * sizeof(float);
}

namespace {
hipError_t dispatch_phases(const ForwardArgs& a, int d, int io_dtype, hipStream_t stream) {
  const bool bf = io_dtype == 1;
  switch (d) {
    case 32: return bf ? launch_phases<32, 2, uint16_t>(a, stream) : launch_phases<32, 2, float>(a, stream);
    case 64: return bf ? launch_phases<64, 2, uint16_t>(a, stream) : launch_phases<64, 2, float>(a, stream);
    case 96: return bf ? launch_phases<96, 3, uint16_t>(a, stream) : launch_phases<96, 3, float>(a, stream);
    case 128: return bf ? launch_phases<128, 4, uint16_t>(a, stream) : launch_phases<128, 4, float>(a, stream);
    default: return hipErrorInvalidValue;
  }
}
}  // namespace

hipError_t launch_two_phase(const ForwardArgs& a, int d, int io_dtype, hipStream_t stream) {
  ForwardArgs args = a;
  args.n_seg = 1;
  args.seg_blocks = (a.T + C - 1) / C;
  args.seg_A = nullptr;
  args.seg_S = nullptr;
  args.seg_PQ = nullptr;
  args.seg_zkey = nullptr;
  return dispatch_phases(args, d, io_dtype, stream);
}

// ---------------------------------------------------------------------------------- time-parallel mode
// Segments are sized so that heads x segments gives every compute unit about four workgroups on long
// sequences (segments of at least 16 blocks: the map pass costs two extra sweeps of S whatever the segment
// count) and one workgroup on short ones (segments of at least 2 blocks).  Measured at d = 64: 16 heads are
// fastest with 16 segments from T = 512 (0.10 ms, fused block kernel 0.16 ms) to T = 4096 (0.20 ms), 64 heads
// with 4 segments up to T = 1024 and 8 at T = 2048, 128 heads with 2-4.
// From d = 96 the A scan holds two workgroups per compute unit and the d^3 work per segment (boundary inverse,
// composition of the maps) weighs four to eight times more: 512 pairs (one resident round) and segments of at
// least 32 blocks.  Measured at d = 128, 16 heads: T = 32768 2.00 ms with 32 segments against 2.28 with 64 and
// 2.52 with 24 (three quarters of a round take as long as a whole one); T = 8192 0.65 with 16 against 0.73 with
// 32; 8 heads, T = 32768: 1.22 with 64 against 1.59 with 128; d = 96, 16 heads, T = 32768: 1.52 against 1.84.
// With the options (`general`: the A chain runs on the option kernel, three workgroups per compute unit at
// d = 64) a resident round is 768 pairs at d = 64, and the longer chain favours segments of 32 blocks there too:
// 16 heads, T = 131072: 3.04 ms with 48 segments against 3.15 with 64; T = 16384: 0.49 with 32 against 0.55
// with 64; 8 heads, T = 65536: 0.90 with 96 against 1.00 with 128.
SegmentPlan plan_segments(int n_heads, int T, int d, bool general, int requested) {
  const int nblk = (T + C - 1) / C;
  int ns = requested;
  if (ns <= 0) {
    const int heads = n_heads < 1 ? 1 : n_heads;
    const bool wide = d >= 96;
    const bool long_chain = wide || (general && d == 64);
    const int most_pairs = wide ? 512 : (long_chain ? 768 : 1024);
    const int by_chip = most_pairs / heads;
    const int by_length = nblk / (long_chain ? 32 : 16);
    int one_per_cu = 256 / heads;
    if (one_per_cu > nblk / 2) one_per_cu = nblk / 2;
    ns = by_length > one_per_cu ? by_length : one_per_cu;
    if (ns > by_chip) ns = by_chip;
    // Whole rounds of 256 pairs: a compute unit that gets a second workgroup of the S-row kernels while others
    // have one takes twice as long over it.  24 heads, d = 64, T = 16384: 21 segments (504 pairs) 0.57 ms, 22
    // segments 0.68; T = 4096: 16 segments (384 pairs) 0.23, 21 segments 0.22, 10 segments 0.23, 11 segments 0.30;
    // d = 128, T = 8192: 16 segments 1.05, 21 segments 0.92.
    if (heads <= 128 && ns * heads > 256) {
      int rounds = (ns * heads + 128) / 256;
      if (rounds > most_pairs / 256) rounds = most_pairs / 256;
      ns = 256 * rounds / heads;
    }
  }
  if (ns > 256) ns = 256;
  if (ns > nblk) ns = nblk;
  if (ns < 1) ns = 1;
  SegmentPlan p;
  p.seg_blocks = nblk > 0 ? (nblk + ns - 1) / ns : 0;
  p.n_seg = nblk > 0 ? (nblk + p.seg_blocks - 1) / p.seg_blocks : 1;  // no empty segment
  return p;
}

namespace {
// workspace of the time-parallel mode, in floats, after the two-phase region
struct TpLayout {
  size_t gram, seg_A, seg_PQ, seg_S, key_part, seg_zkey, total;
};
TpLayout tp_layout(int n_heads, int T, int d, int d_v, int n_seg) {
  const int nblk = (T + C - 1) / C;
  const size_t mats = static_cast<size_t>(n_heads) * n_seg * d * d;  // one d x d float matrix per (head, seg)
  const size_t smats = static_cast<size_t>(n_heads) * n_seg * d_v * d;  // one d_v x d matrix (S, Q) per (head, seg)
  TpLayout l;
  size_t off = static_cast<size_t>(n_heads) * head_stride(nblk, d);
  off = (off + 3) & ~static_cast<size_t>(3);  // 16-byte alignment
  l.gram = off;   off += 2 * mats;            // float64
  l.seg_A = off;  off += mats;
  l.seg_PQ = off; off += mats + smats;
  l.seg_S = off;  off += smats;
  const size_t vecs = static_cast<size_t>(n_heads) * n_seg * d;      // one d-vector per (head, seg)
  l.key_part = off; off += 2 * vecs;          // float64
  l.seg_zkey = off; off += vecs;
  off = (off + 3) & ~static_cast<size_t>(3);
  l.total = off;
  return l;
}
}  // namespace

size_t time_parallel_workspace_bytes(int n_heads, int T, int d, int d_v, bool general, int requested_segments) {
  const SegmentPlan p = plan_segments(n_heads, T, d, general, requested_segments);
  if (p.n_seg <= 1) return two_phase_workspace_bytes(n_heads, T, d);
  return tp_layout(n_heads, T, d, d_v, p.n_seg).total * sizeof(float);
}

hipError_t launch_time_parallel(const ForwardArgs& a, int d, int io_dtype, int requested_segments,
                                hipStream_t stream) {
  const SegmentPlan p = plan_segments(a.n_heads, a.T, d, runs_on_option_kernel(a), requested_segments);
  if (p.n_seg <= 1) return launch_two_phase(a, d, io_dtype, stream);
  const TpLayout l = tp_layout(a.n_heads, a.T, d, a.d_v > 0 ? a.d_v : d, p.n_seg);
  ForwardArgs args = a;
  args.n_seg = p.n_seg;
  args.seg_blocks = p.seg_blocks;
  double* G = reinterpret_cast<double*>(a.ws + l.gram);
  args.seg_A = a.ws + l.seg_A;
  args.seg_PQ = a.ws + l.seg_PQ;
  args.seg_S = a.ws + l.seg_S;
  hipError_t err = launch_gram(args, d, io_dtype, G, stream);
  if (err != hipSuccess) return err;
  err = launch_boundary(args, d, G, a.ws + l.seg_A, stream);
  if (err != hipSuccess) return err;
  if (a.normalise_output != 0 || a.zkey_T != nullptr) {   // the key sum every segment starts with
    float* seg_zkey = a.ws + l.seg_zkey;
    err = launch_keysum(args, d, io_dtype, reinterpret_cast<double*>(a.ws + l.key_part), seg_zkey, stream);
    if (err != hipSuccess) return err;
    args.seg_zkey = seg_zkey;
  }
  return dispatch_phases(args, d, io_dtype, stream);
}

}  // namespace vla
