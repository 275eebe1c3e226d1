// State at the boundaries of time segments, for the time-parallel mode.
//
// Without the identity refresh the inverse penalty matrix is an explicit inverse (paper Section 3.2 and
// eq. (penalty); eq. (sm) is the Sherman-Morrison form of it):  A_t = (A_0^{-1} + sum_{s<=t} u_s u_s^T)^{-1}, with
// u_s = k^_s by default or the caller's penalty directions, normalised and scaled.  The sum is a plain prefix
// sum, so A at the start of every segment follows from one Gram matrix per segment and one d x d inversion, all
// independent of each other; the segments then run the exact rank-1 recurrence concurrently.  The paper
// treats the A loop as sequential (Section 3.4); this goes beyond it and is not valid with the identity
// refresh.  The directions are the float32 numbers the recurrence kernels work with; their outer products (exact
// in float64), the sums and the inversions are float64, so that the boundary matrices are at least as accurate
// as the float32 chain they replace.
//
// The S recurrence is affine in S (eq. (s-update)): S_end = S_start P + Q per segment.  P and Q come from the
// map pass of the S-rows kernel; combine_kernel composes them from left to right.
#include "vla_mfma_util.h"
#include <type_traits>

namespace vla {
namespace {

constexpr int kThreads = 256;

// ------------------------------------------------------------------------------------------ Gram
typedef double d4 __attribute__((ext_vector_type(4)));

// One workgroup (4 waves) per (head, segment); the last segment's matrix is never needed.  Tokens are
// normalised in float32, exactly as the kernels that run the recurrence normalise them (the sum is over the
// directions those kernels use, float32 numbers), and staged through LDS 64 at a time (32 at d = 128); the outer
// products run on the float64 matrix cores (v_mfma_f64_16x16x4_f64: lane l supplies A[i = l % 16][k = l / 16] and
// B[k = l / 16][j = l % 16] and receives D[i = l / 16 + 4 r][j = l % 16] in element r), both operands being the
// same staged tile widened as it is read: a product of two float32 values is exact in float64.  A wave
// holds at most 16 result tiles: up to D = 64 every wave covers the whole matrix and the waves take the
// tokens of a tile in turn (summed through LDS at the end); at D = 128 wave w owns the tile rows w and
// DL/16 - 1 - w from the diagonal on (DL/16 + 1 tiles whatever w: the sum is symmetric, the tiles below the
// diagonal are mirrored at the end).
// DL: the head size of the data; D >= DL: the size the tiles are laid out for.  They differ for d = 96, which
// runs in the d = 128 layout with the columns from 96 on held at zero (the loads, the staging and the final
// stores skip them; three of the four waves then form the products).
template <int D, int DL, typename IO>
__global__ void __launch_bounds__(kThreads, D <= 64 ? 3 : 2) gram_kernel(ForwardArgs a, double* G) {
  static_assert(DL <= D && DL % 16 == 0, "padded layout");
  constexpr int NTI = D / 16;                                // tiles per side
  constexpr int TR = NTI * NTI <= 16 ? NTI : 16 / NTI;       // tile rows per wave
  constexpr int RGW = NTI / TR;                              // waves across the rows
  constexpr int NGW = (kThreads / 64) / RGW;                 // waves across the tokens
  constexpr int TT = D <= 64 ? 64 : 32;                      // tokens per tile
  constexpr int KS = TT / 4;                                 // k-steps (4 tokens) per tile
  constexpr int LDK = D + 16;                                // rows 16 banks apart: conflict-free operand reads
  constexpr int EPT = TT * D / kThreads;                     // elements of the tile each thread stages
  constexpr int TPR = D / EPT;                               // threads per token row
  static_assert(RGW * NGW * 64 == kThreads && KS % NGW == 0 && (TPR == 4 || TPR == 8) && EPT % 4 == 0, "layout");
  // The sum of k^ k^T is symmetric: only the tiles on and above the diagonal are formed (10 of 16 at d = 64,
  // 36 of 64 at d = 128).  Where a wave cannot hold the whole matrix the tile rows are paired so that every
  // wave has the same number of them.
  constexpr bool PAIR = RGW > 1;
  constexpr int NTL = DL / 16;                               // tile rows that hold data
  constexpr int NPT = NTL + 1;                               // tiles of a wave's pair of rows
  static_assert(PAIR ? (NTL % 2 == 0 && NTL / 2 <= RGW && NGW == 1) : (RGW == 1 && D == DL),
                "row w pairs with row NTL - 1 - w; otherwise every wave covers the whole matrix");
  __shared__ __align__(16) float ktb[2][TT * LDK];   // double-buffered: one barrier per tile
  static_assert(NGW == 1 || 2 * TT * LDK * sizeof(float) >= D * D * sizeof(double),
                "the final sum over the waves reuses the tile buffers");
  double* const red = reinterpret_cast<double*>(&ktb[0][0]);

  const int head = blockIdx.x / a.n_seg;
  const int seg = blockIdx.x - head * a.n_seg;
  if (seg == a.n_seg - 1) return;
  const int tid = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63;
  const int c = lane & 15;
  const int g = lane >> 4;
  const int tgrp = w / RGW;     // which k-steps
  const int tb = seg * a.seg_blocks * C;
  const int te = min(a.T, tb + a.seg_blocks * C);
  // the directions the penalty matrix accumulates: the caller's u (scaled after normalisation), else the keys
  const bool has_u = a.u != nullptr;
  const IO* kh = static_cast<const IO*>(has_u ? a.u : a.k) + static_cast<size_t>(head) * static_cast<size_t>(a.T) * DL;
  const float eps = a.eps;
  const float scale = has_u ? a.u_scale : 1.0f;
  const int srow = tid / TPR;
  const int scol = (tid % TPR) * EPT;

  d4 acc[PAIR ? 1 : TR][PAIR ? 1 : NTI];   // every wave covers the whole matrix, or whole tile rows
  d4 pacc[PAIR ? NPT : 1];                 // paired rows: row w from its diagonal tile on, then row NTL - 1 - w
#pragma unroll
  for (int i = 0; i < (PAIR ? 1 : TR); ++i)
#pragma unroll
    for (int j = 0; j < (PAIR ? 1 : NTI); ++j) acc[i][j] = d4{0, 0, 0, 0};
#pragma unroll
  for (int i = 0; i < (PAIR ? NPT : 1); ++i) pacc[i] = d4{0, 0, 0, 0};

  // Fragments of the next PF tiles are kept in flight in raw form (a few registers each): with a thousand
  // workgroups streaming at once the memory latency is several tiles' worth of work.
  constexpr int PF = 2;   // what the register file allows next to the accumulator registers
  RawRow<IO, EPT> raw[PF];
  auto fetch = [&](int t0, RawRow<IO, EPT>& o) {
    const int t = t0 + srow;
    if (D == DL || scol < DL) o.load(kh + static_cast<size_t>(t < te ? t : te - 1) * DL + scol);
  };
  // stage: k^ = k / max(||k||, eps) as the recurrence kernels form it (float32: hardware reciprocal square
  // root, one Newton step); rows past the end are zero
  auto stage = [&](int t0, const RawRow<IO, EPT>& o, float* kt) {
    const int t = t0 + srow;
    float x[EPT];
    o.unpack(x);
    if (D != DL && scol >= DL) {
#pragma unroll
      for (int e = 0; e < EPT; ++e) x[e] = 0.0f;
    }
    if (a.feature_map && !has_u && (D == DL || scol < DL)) {   // ELU(x) + 1 on keys
#pragma unroll
      for (int e = 0; e < EPT; ++e) x[e] = elu_plus_one(x[e]);
    }
    float ss = 0.0f;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      x[e] = t < te ? x[e] : 0.0f;
      ss = fmaf(x[e], x[e], ss);
    }
#pragma unroll
    for (int off = TPR / 2; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
    const float sm = fmaxf(ss, eps * eps);
    float rn = __builtin_amdgcn_rsqf(sm);
    rn = rn * fmaf(-0.5f * sm * rn, rn, 1.5f) * scale;
#pragma unroll
    for (int e = 0; e < EPT; e += 4)
      *reinterpret_cast<f4*>(&kt[srow * LDK + scol + e]) = f4{x[e] * rn, x[e + 1] * rn, x[e + 2] * rn, x[e + 3] * rn};
  };
  // paired rows, for the wave W (a compile-time copy of w): tiles (W, W..NTL-1) then (R1, R1..NTL-1)
  auto pair_products = [&](auto wtag, const float* kt) {
    constexpr int W = decltype(wtag)::value;
    constexpr int R1 = NTL - 1 - W;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      const float* row = &kt[(4 * kk + g) * LDK + c];
      double bv[NTL];
#pragma unroll
      for (int j = W; j < NTL; ++j) bv[j] = static_cast<double>(row[16 * j]);
#pragma unroll
      for (int j = W; j < NTL; ++j)
        pacc[j - W] = __builtin_amdgcn_mfma_f64_16x16x4f64(bv[W], bv[j], pacc[j - W], 0, 0, 0);
#pragma unroll
      for (int j = R1; j < NTL; ++j)
        pacc[NTL - W + j - R1] = __builtin_amdgcn_mfma_f64_16x16x4f64(bv[R1], bv[j], pacc[NTL - W + j - R1], 0, 0, 0);
    }
  };
  // element r of the tile (i, j) is G[16 i + g + 4 r][16 j + c]; its mirror image fills the tile (j, i)
  auto pair_store = [&](auto wtag, double* Gh) {
    constexpr int W = decltype(wtag)::value;
    constexpr int R1 = NTL - 1 - W;
    auto put = [&](int i, int j, const d4& t) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int row = 16 * i + g + 4 * r, col = 16 * j + c;
        Gh[row * DL + col] = t[r];
        if (j > i) Gh[col * DL + row] = t[r];
      }
    };
#pragma unroll
    for (int j = W; j < NTL; ++j) put(W, j, pacc[j - W]);
#pragma unroll
    for (int j = R1; j < NTL; ++j) put(R1, j, pacc[NTL - W + j - R1]);
  };
  // the wave's own copy of the two above (w is uniform over the wave)
  auto for_my_rows = [&](auto&& f) {
    if constexpr (PAIR) {
      if (w == 0) f(std::integral_constant<int, 0>{});
      if (w == 1 && NTL >= 4) f(std::integral_constant<int, (NTL >= 4 ? 1 : 0)>{});
      if (w == 2 && NTL >= 6) f(std::integral_constant<int, (NTL >= 6 ? 2 : 0)>{});
      if (w == 3 && NTL >= 8) f(std::integral_constant<int, (NTL >= 8 ? 3 : 0)>{});
    }
  };
  auto products = [&](const float* kt) {
    if constexpr (PAIR) {
      for_my_rows([&](auto wtag) { pair_products(wtag, kt); });
    } else {
#pragma unroll
      for (int kk = tgrp; kk < KS; kk += NGW) {
        const float* row = &kt[(4 * kk + g) * LDK + c];
        double bv[NTI];
#pragma unroll
        for (int j = 0; j < NTI; ++j) bv[j] = static_cast<double>(row[16 * j]);
#pragma unroll
        for (int i = 0; i < TR; ++i)
#pragma unroll
          for (int j = i; j < NTI; ++j)   // tiles below the diagonal are mirrored at the end
            acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(bv[i], bv[j], acc[i][j], 0, 0, 0);
      }
    }
  };
#pragma unroll
  for (int u = 0; u < PF; ++u)
    if (tb + u * TT < te) fetch(tb + u * TT, raw[u]);
  for (int t0 = tb; t0 < te; t0 += PF * TT) {
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      const int tu = t0 + u * TT;
      if (tu < te) {   // uniform over the workgroup
        float* kt = ktb[u & 1];
        stage(tu, raw[u], kt);
        // the buffer written here was last read two tiles ago, and every wave has passed the barrier of the
        // tile in between since then
        __syncthreads();
        if (tu + PF * TT < te) fetch(tu + PF * TT, raw[u]);
        products(kt);
      }
    }
  }

  double* Gh = G + static_cast<size_t>(blockIdx.x) * DL * DL;
  if constexpr (PAIR) {
    for_my_rows([&](auto wtag) { pair_store(wtag, Gh); });
  } else {
    // element r of tile (i, j) is G[16 i + g + 4 r][16 j + c]; the waves' partial sums meet in LDS
    __syncthreads();   // every wave is done with the tile buffers
    for (int gi = 0; gi < NGW; ++gi) {
      if (tgrp == gi) {
#pragma unroll
        for (int i = 0; i < TR; ++i)
#pragma unroll
          for (int j = i; j < NTI; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int o = (16 * i + g + 4 * r) * D + 16 * j + c;
              red[o] = gi == 0 ? acc[i][j][r] : red[o] + acc[i][j][r];
            }
      }
      __syncthreads();
    }
    for (int o = tid; o < D * D; o += kThreads) {
      const int row = o / D, col = o - row * D;
      Gh[o] = row / 16 > col / 16 ? red[col * D + row] : red[o];   // tile below the diagonal: mirror
    }
  }
}

// In-place inclusive prefix sum of the Gram matrices over the segments of a head, one thread per element:
// afterwards G[h][s] = sum over segments 0..s.
__global__ void __launch_bounds__(kThreads) gram_prefix_kernel(double* G, int n_heads, int n_seg, int dd) {
  const long long e = static_cast<long long>(blockIdx.x) * kThreads + threadIdx.x;
  if (e >= static_cast<long long>(n_heads) * dd) return;
  const int head = static_cast<int>(e / dd);
  double* p = G + (static_cast<size_t>(head) * n_seg) * dd + (e - static_cast<long long>(head) * dd);
  double run = 0.0;
  const int n = n_seg - 1;   // the last segment's matrix is never needed
  // sixteen loads in flight at a time: the chain is as long as the memory latency times the trips it makes
  constexpr int U = 16;
  for (int s = 0; s < n; s += U) {
    double x[U];
#pragma unroll
    for (int i = 0; i < U; ++i) x[i] = s + i < n ? p[static_cast<size_t>(s + i) * dd] : 0.0;
#pragma unroll
    for (int i = 0; i < U; ++i) {
      run += x[i];
      if (s + i < n) p[static_cast<size_t>(s + i) * dd] = run;
    }
  }
}

// ------------------------------------------------------------------------------------------ key sums
// Normalised read-out (eq. (output)): zkey_t = zkey_0 + sum_{s<=t} k_s with k_s the key as used before its L2
// normalisation (after the feature map).  Per (head, segment) the sum of its keys, in float64; a thread adds eight
// consecutive columns of every RG-th token, the row groups are summed through LDS.
template <int D, typename IO>
__global__ void __launch_bounds__(kThreads) keysum_kernel(ForwardArgs a, double* part) {
  constexpr int EPT = 8;                 // consecutive columns per thread: one 16- or 32-byte piece of a row
  constexpr int TPR = D / EPT;           // threads per token row
  constexpr int RG = kThreads / TPR;     // rows in flight per pass (the last groups idle when 256 / TPR is no integer)
  __shared__ double red[RG][D];
  const int head = blockIdx.x / a.n_seg;
  const int seg = blockIdx.x - head * a.n_seg;
  const int rg = threadIdx.x / TPR;
  const int j0 = (threadIdx.x % TPR) * EPT;
  const int tb = seg * a.seg_blocks * C;
  const int te = min(a.T, tb + a.seg_blocks * C);
  const IO* kh = static_cast<const IO*>(a.k) + static_cast<size_t>(head) * static_cast<size_t>(a.T) * D;
  double sum[EPT];
#pragma unroll
  for (int e = 0; e < EPT; ++e) sum[e] = 0.0;
  if (rg < RG) {
    for (int t = tb + rg; t < te; t += RG) {
      RawRow<IO, EPT> raw;
      raw.load(kh + static_cast<size_t>(t) * D + j0);
      float x[EPT];
      raw.unpack(x);
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        if (a.feature_map) x[e] = elu_plus_one(x[e]);
        sum[e] += static_cast<double>(x[e]);
      }
    }
#pragma unroll
    for (int e = 0; e < EPT; ++e) red[rg][j0 + e] = sum[e];
  }
  __syncthreads();
  for (int j = threadIdx.x; j < D; j += kThreads) {
    double total = 0.0;
    for (int r = 0; r < RG; ++r) total += red[r][j];
    part[static_cast<size_t>(blockIdx.x) * D + j] = total;
  }
}
// seg_zkey[h][s] = zkey0[h] + the sums of the segments before s, one thread per (head, column)
__global__ void __launch_bounds__(kThreads) keysum_prefix_kernel(const double* part, const float* zkey0,
                                                                 float* seg_zkey, int n_heads, int n_seg, int d) {
  const long long e = static_cast<long long>(blockIdx.x) * kThreads + threadIdx.x;
  if (e >= static_cast<long long>(n_heads) * d) return;
  const int head = static_cast<int>(e / d);
  const int j = static_cast<int>(e - static_cast<long long>(head) * d);
  double run = zkey0 ? static_cast<double>(zkey0[e]) : 0.0;
  const size_t base = static_cast<size_t>(head) * n_seg * d + j;
  constexpr int U = 16;   // loads in flight
  for (int s = 0; s < n_seg; s += U) {
    double x[U];
#pragma unroll
    for (int i = 0; i < U; ++i) x[i] = s + i < n_seg ? part[base + static_cast<size_t>(s + i) * d] : 0.0;
#pragma unroll
    for (int i = 0; i < U; ++i) {
      if (s + i < n_seg) seg_zkey[base + static_cast<size_t>(s + i) * d] = static_cast<float>(run);
      run += x[i];
    }
  }
}

// ------------------------------------------------------------------------------------------ boundary
// Gauss-Jordan inverse, in place, of a symmetric positive definite D x D matrix spread over the workgroup's
// registers (no pivoting needed for such a matrix) in the result layout of the float64 matrix instruction:
// wave w holds the tile row w, lane (g, c) of it acc[tj][r] = M[16 w + g + 4 r][16 tj + c].
//
// The sweep eliminates KB = 4 pivots at a time.  With P the pivot indices of a step, B = M[P][P], C = M[:, P]
// and R = M[P, :], the in-place step is  M <- M - C' R'  with
//   C'[i] = C[i] (i not in P),  C'[P] = B - I;     R'[:, j] = B^{-1} R[:, j] (j not in P),  R'[:, P] = I + B^{-1}
// which is the usual block sweep (Schur complement off the pivot rows and columns, -C B^{-1} in the pivot
// columns, B^{-1} R in the pivot rows, B^{-1} in the pivot block) written so that every element takes the same
// rank-4 update: one v_mfma_f64_16x16x4_f64 per 16 x 16 tile and step.  The pivot rows are not fetched at
// all: after the earlier steps the not yet eliminated part of M is a Schur complement (symmetric) and the
// eliminated part of a pivot row is minus the transposed column, so R[a][j] = C[j][a] for j after P and -C[j][a]
// for j before it.  Only the four pivot columns go through LDS (the lanes that hold them copy their registers
// out, with the identity already subtracted from the pivot block), double-buffered: one barrier per step.
// Every lane factors the 4 x 4 block B = L diag(dd) L^T for itself in registers and solves for the one row of
// B^{-1} it needs (row g: a lane supplies R'[g][16 tj + c] as the B operand of tile tj and C'[16 w + c][g] as
// the A operand); the pivot columns get theirs from the identity x = e_e - B^{-1} e_e that the stored B - I gives
// them.  A lane reads 4 tj + 15 doubles from LDS per step; with the matrix spread as a quarter of a column per
// thread and the update on the vector units it read D + 14, and the LDS pipe was what the sweep waited for
// (d = 128, 496 matrices: 0.18 ms).
template <int D>
struct SpdInverse {
  static constexpr int NTL = D / 16;        // tile rows (one wave each) and tile columns
  static constexpr int NT = 64 * NTL;       // 4 D threads
  static constexpr int KB = 4;              // pivots per step: the contraction length of the matrix instruction
  static constexpr int STRIDE = D;          // doubles per pivot column
  static constexpr int LDS_DOUBLES = 2 * KB * STRIDE;
  double* colp;                             // LDS [2][KB][STRIDE]
  static __device__ __forceinline__ double recip(double d) {   // hardware estimate refined twice: full precision
    const double y = __builtin_amdgcn_rcp(d);
    const double y1 = y * fma(-d, y, 2.0);
    return y1 * fma(-d, y1, 2.0);
  }
  __device__ __forceinline__ void run(d4 (&acc)[NTL]) const {
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int c = lane & 15;
    const int g = lane >> 4;
#pragma unroll
    for (int tp = 0; tp < NTL; ++tp) {       // the tile column that holds the pivots
      for (int ps = 0; ps < 4; ++ps) {       // its columns 4 ps .. 4 ps + 3
        const int p0 = 16 * tp + KB * ps;
        double* cp = colp + (ps & 1) * (KB * STRIDE);
        if ((c >> 2) == ps) {                // this lane's column of tile tp is pivot e of the step
          double* mine = cp + (c & 3) * STRIDE + 16 * w + g;
#pragma unroll
          for (int r = 0; r < 4; ++r) mine[4 * r] = acc[tp][r] - ((w == tp && g + 4 * r == c) ? 1.0 : 0.0);
        }
        __syncthreads();
        // B = L diag(dd) L^T (unit lower triangular L, no pivoting: B is symmetric positive definite), every
        // lane for itself in registers; lo[a][c] holds B's lower triangle, then t = L diag(dd) below the diagonal
        double lo[KB][KB], l[KB][KB], inv[KB];
#pragma unroll
        for (int a = 0; a < KB; ++a)
#pragma unroll
          for (int k = 0; k <= a; ++k) {
            const double x = cp[k * STRIDE + p0 + a];
            lo[a][k] = (a == k) ? x + 1.0 : x;
          }
#pragma unroll
        for (int k = 0; k < KB; ++k) {
          // column k: t[a][k] = B[a][k] - sum_{i<k} l[a][i] t[k][i];  dd_k = t[k][k];  l[a][k] = t[a][k] / dd_k
#pragma unroll
          for (int a = k; a < KB; ++a)
#pragma unroll
            for (int i = 0; i < k; ++i) lo[a][k] = fma(-l[a][i], lo[k][i], lo[a][k]);
          inv[k] = recip(lo[k][k]);
#pragma unroll
          for (int a = k + 1; a < KB; ++a) l[a][k] = lo[a][k] * inv[k];
        }
        // y = row g of B^{-1} (= column g: B is symmetric), by the two triangular solves on e_g
        double y[KB];
#pragma unroll
        for (int a = 0; a < KB; ++a) y[a] = (a == g) ? 1.0 : 0.0;
#pragma unroll
        for (int a = 1; a < KB; ++a)
#pragma unroll
          for (int k = 0; k < a; ++k) y[a] = fma(-l[a][k], y[k], y[a]);
#pragma unroll
        for (int a = 0; a < KB; ++a) y[a] *= inv[a];
#pragma unroll
        for (int a = KB - 2; a >= 0; --a)
#pragma unroll
          for (int k = a + 1; k < KB; ++k) y[a] = fma(-l[k][a], y[k], y[a]);
        const double cv = cp[g * STRIDE + 16 * w + c];   // C'[16 w + c][g]
        // x = (B^{-1} (M[j][P])^T)[g] for the lane's column j of every tile; then R'[g][j]:
        //   j after the pivots:   R[:, j] = +M[j][P]^T            -> x
        //   j before the pivots:  R[:, j] = -M[j][P]^T            -> -x
        //   j = pivot e:          the column holds (B - I)[:, e]  -> x = (e_e - B^{-1} e_e)[g],  R' = 2 [e = g] - x
#pragma unroll
        for (int tj = 0; tj < NTL; ++tj) {
          const int j = 16 * tj + c;
          double x = y[0] * cp[j];
#pragma unroll
          for (int k = 1; k < KB; ++k) x = fma(y[k], cp[k * STRIDE + j], x);
          const double rr = (j >= p0 + KB) ? x : ((j - p0 == g) ? 2.0 - x : -x);
          acc[tj] = __builtin_amdgcn_mfma_f64_16x16x4f64(cv, -rr, acc[tj], 0, 0, 0);
        }
      }
    }
  }
};

// One workgroup per (head, segment): seg_A = inverse(inverse(A0) + sum of the Gram matrices before it),
// G holding the prefix sums.
// DL: the head size of the data; D >= DL: the size the inversion is laid out for (d = 96 runs in the d = 128
// layout: the matrix is bordered with an identity block, whose inverse is itself).
template <int D, int DL>
__global__ void __launch_bounds__(SpdInverse<D>::NT, D <= 64 ? 4 : 2) boundary_kernel(ForwardArgs a, const double* G, float* seg_A) {
  static_assert(DL <= D, "padded layout");
  constexpr int NTL = SpdInverse<D>::NTL;
  constexpr int NT = SpdInverse<D>::NT;
  __shared__ __align__(16) double colp[SpdInverse<D>::LDS_DOUBLES];

  const int head = blockIdx.x / a.n_seg;
  const int seg = blockIdx.x - head * a.n_seg;
  const int lane = threadIdx.x & 63;
  const int c = lane & 15;
  const int i0 = 16 * (threadIdx.x >> 6) + (lane >> 4);   // acc[tj][r] = M[i0 + 4 r][16 tj + c]
  const float* A0 = a.A0 ? a.A0 + static_cast<size_t>(head) * DL * DL : nullptr;
  float* out = seg_A + static_cast<size_t>(blockIdx.x) * DL * DL;
  const float diag = 1.0f / a.lambda0;   // the same float32 value the first segment starts from

  if (seg == 0) {   // the first segment starts from the caller's A0, bit for bit
    for (int e = threadIdx.x; e < DL * DL; e += NT) out[e] = A0 ? A0[e] : (e / DL == e % DL ? diag : 0.0f);
    return;
  }
  auto data = [&](int i, int j) { return D == DL || (i < DL && j < DL); };   // inside the DL x DL matrix
  const SpdInverse<D> inv{colp};
  d4 acc[NTL];
  if (A0) {
#pragma unroll
    for (int tj = 0; tj < NTL; ++tj)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int i = i0 + 4 * r, j = 16 * tj + c;
        acc[tj][r] = data(i, j) ? 0.5 * (static_cast<double>(A0[i * DL + j]) + static_cast<double>(A0[j * DL + i]))
                                : (i == j ? 1.0 : 0.0);
      }
    inv.run(acc);
    __syncthreads();   // the pivot buffers are reused by the second inversion
  } else {
#pragma unroll
    for (int tj = 0; tj < NTL; ++tj)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int i = i0 + 4 * r, j = 16 * tj + c;
        acc[tj][r] = (i == j) ? (data(i, j) ? 1.0 / static_cast<double>(diag) : 1.0) : 0.0;
      }
  }
  // G holds inclusive prefix sums: G[head][seg - 1] covers every token before this segment
  const double* Gh = G + (static_cast<size_t>(blockIdx.x) - 1) * DL * DL;
#pragma unroll
  for (int tj = 0; tj < NTL; ++tj)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int i = i0 + 4 * r, j = 16 * tj + c;
      if (data(i, j)) acc[tj][r] += Gh[i * DL + j];
    }
  inv.run(acc);
  // The inverse of a symmetric matrix is symmetric up to rounding; store the lower triangle's values on both
  // sides so that the float32 matrix the recurrence starts from is exactly symmetric.
#pragma unroll
  for (int tj = 0; tj < NTL; ++tj)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int i = i0 + 4 * r, j = 16 * tj + c;
      const float v = static_cast<float>(acc[tj][r]);
      if (i >= j && data(i, j)) {
        out[i * DL + j] = v;
        out[j * DL + i] = v;
      }
    }
}

// ------------------------------------------------------------------------------------------ combine
// x <- x P_s + Q_s for s = 0 .. n_seg-2, every intermediate written out as the start state of segment s+1.
// One workgroup per (head, 16-row slab of S), one wave per 16-column slice of the result: each wave keeps the
// whole slab x as accumulator tiles, xt[b][r] = S[row0 + c][16b + 4g + r] (the layout the S-rows kernel loads
// its start state in; the contraction index is taken in the order k = 16b + 4g + r so that a tile feeds
// straight back as the MFMA B operand), computes its own slice of x P + Q and hands it to the other waves
// through LDS.  The chain is sequential in s and short per step, so the operands of the next three
// segments are kept in flight in rotating register sets.
// S has a.d_v rows (value heads of another size than the key heads: more or fewer slabs per head, P stays D x D).
template <int D>
__global__ void __launch_bounds__(64 * (D / 16)) combine_kernel(ForwardArgs a, float* seg_S) {
  constexpr int NB = D / 16;
  constexpr int LDX = D + 4;
  constexpr int LA = 3;   // segments of lookahead
  __shared__ __align__(16) float xs[2][16 * LDX];
  const int dv = a.d_v > 0 ? a.d_v : D;
  const int nbv = dv / 16;                       // slabs per head
  const size_t ssz = static_cast<size_t>(dv) * D;            // floats of S and of Q
  const size_t pqsz = static_cast<size_t>(D) * D + ssz;      // floats of one segment's P then Q
  const int head = blockIdx.x / nbv;
  const int row0 = (blockIdx.x - head * nbv) * 16;
  const int jb = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // column slice of this wave
  const int lane = threadIdx.x & 63;
  const int c = lane & 15;
  const int g = lane >> 4;
  const size_t hbase = static_cast<size_t>(head) * a.n_seg;
  const int ro = (row0 + c) * D + 4 * g;   // this lane's float4 inside a d x d matrix, plus 16 b
  const int n = a.n_seg - 1;               // steps

  struct Seg {
    float pa[NB][4];   // P[16b + 4g + r][16 jb + c]
    f4 q;              // Q[row0 + c][16 jb + 4g ..]
  };
  auto load = [&](int s, Seg& o) {
    const float* P = a.seg_PQ + (hbase + s) * pqsz;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int r = 0; r < 4; ++r) o.pa[b][r] = P[(16 * b + 4 * g + r) * D + 16 * jb + c];
    o.q = *reinterpret_cast<const f4*>(P + D * D + ro + 16 * jb);
  };

  f4 xt[NB];
  {
    const float* S0 = a.S0 ? a.S0 + static_cast<size_t>(head) * ssz : nullptr;
#pragma unroll
    for (int b = 0; b < NB; ++b) xt[b] = S0 ? *reinterpret_cast<const f4*>(S0 + ro + 16 * b) : f4{0, 0, 0, 0};
    const f4 mine = S0 ? *reinterpret_cast<const f4*>(S0 + ro + 16 * jb) : f4{0, 0, 0, 0};
    *reinterpret_cast<f4*>(seg_S + hbase * ssz + ro + 16 * jb) = mine;
  }

  auto step = [&](int s, const Seg& o) {
    f4 nx = o.q;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int r = 0; r < 4; ++r) nx = mfma16(o.pa[b][r], xt[b][r], nx);
    *reinterpret_cast<f4*>(seg_S + (hbase + s + 1) * ssz + ro + 16 * jb) = nx;
    float* x = xs[s & 1];
    *reinterpret_cast<f4*>(&x[c * LDX + 16 * jb + 4 * g]) = nx;
    __syncthreads();
#pragma unroll
    for (int b = 0; b < NB; ++b) xt[b] = lds4(&x[c * LDX + 16 * b + 4 * g]);
  };

  Seg buf[LA + 1];
#pragma unroll
  for (int u = 0; u < LA; ++u)
    if (u < n) load(u, buf[u]);
  for (int s = 0; s < n; s += LA + 1) {
#pragma unroll
    for (int u = 0; u <= LA; ++u) {
      if (s + u < n) {   // uniform over the workgroup
        if (s + u + LA < n) load(s + u + LA, buf[(u + LA) % (LA + 1)]);
        step(s + u, buf[u]);
      }
    }
  }
}

template <int D, int DL = D>
hipError_t launch_boundary_d(const ForwardArgs& a, const double* G, float* seg_A, hipStream_t stream) {
  ForwardArgs args = a;
  void* params[] = {&args, &G, &seg_A};
  return hipLaunchKernel(reinterpret_cast<const void*>(&boundary_kernel<D, DL>), dim3(a.n_heads * a.n_seg),
                         dim3(SpdInverse<D>::NT), params, 0, stream);
}
template <int D, typename IO, int DL = D>
hipError_t launch_gram_d(const ForwardArgs& a, double* G, hipStream_t stream) {
  ForwardArgs args = a;
  void* params[] = {&args, &G};
  hipError_t err = hipLaunchKernel(reinterpret_cast<const void*>(&gram_kernel<D, DL, IO>),
                                   dim3(a.n_heads * a.n_seg), dim3(kThreads), params, 0, stream);
  if (err != hipSuccess) return err;
  int nh = a.n_heads, ns = a.n_seg, dd = DL * DL;
  void* p2[] = {&G, &nh, &ns, &dd};
  const long long elems = static_cast<long long>(nh) * dd;
  return hipLaunchKernel(reinterpret_cast<const void*>(&gram_prefix_kernel),
                         dim3(static_cast<unsigned>((elems + kThreads - 1) / kThreads)), dim3(kThreads), p2, 0,
                         stream);
}
template <int D>
hipError_t launch_combine_d(const ForwardArgs& a, float* seg_S, hipStream_t stream) {
  ForwardArgs args = a;
  void* params[] = {&args, &seg_S};
  const int dv = a.d_v > 0 ? a.d_v : D;
  return hipLaunchKernel(reinterpret_cast<const void*>(&combine_kernel<D>), dim3(a.n_heads * (dv / 16)),
                         dim3(64 * (D / 16)), params, 0, stream);
}

}  // namespace

namespace {
template <int D, typename IO>
hipError_t launch_keysum_d(const ForwardArgs& a, double* part, float* seg_zkey, hipStream_t stream) {
  ForwardArgs args = a;
  void* params[] = {&args, &part};
  hipError_t err = hipLaunchKernel(reinterpret_cast<const void*>(&keysum_kernel<D, IO>),
                                   dim3(a.n_heads * a.n_seg), dim3(kThreads), params, 0, stream);
  if (err != hipSuccess) return err;
  const double* cpart = part;
  const float* z0 = a.zkey0;
  int nh = a.n_heads, ns = a.n_seg, d = D;
  void* p2[] = {&cpart, &z0, &seg_zkey, &nh, &ns, &d};
  const long long elems = static_cast<long long>(nh) * d;
  return hipLaunchKernel(reinterpret_cast<const void*>(&keysum_prefix_kernel),
                         dim3(static_cast<unsigned>((elems + kThreads - 1) / kThreads)), dim3(kThreads), p2, 0,
                         stream);
}
}  // namespace

hipError_t launch_keysum(const ForwardArgs& a, int d, int io_dtype, double* part, float* seg_zkey,
                         hipStream_t stream) {
  const bool bf = io_dtype == 1;
  switch (d) {
    case 32: return bf ? launch_keysum_d<32, uint16_t>(a, part, seg_zkey, stream)
                       : launch_keysum_d<32, float>(a, part, seg_zkey, stream);
    case 64: return bf ? launch_keysum_d<64, uint16_t>(a, part, seg_zkey, stream)
                       : launch_keysum_d<64, float>(a, part, seg_zkey, stream);
    case 96: return bf ? launch_keysum_d<96, uint16_t>(a, part, seg_zkey, stream)
                       : launch_keysum_d<96, float>(a, part, seg_zkey, stream);
    case 128: return bf ? launch_keysum_d<128, uint16_t>(a, part, seg_zkey, stream)
                        : launch_keysum_d<128, float>(a, part, seg_zkey, stream);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_gram(const ForwardArgs& a, int d, int io_dtype, double* G, hipStream_t stream) {
  const bool bf = io_dtype == 1;
  switch (d) {
    case 32: return bf ? launch_gram_d<32, uint16_t>(a, G, stream) : launch_gram_d<32, float>(a, G, stream);
    case 64: return bf ? launch_gram_d<64, uint16_t>(a, G, stream) : launch_gram_d<64, float>(a, G, stream);
    case 96: return bf ? launch_gram_d<128, uint16_t, 96>(a, G, stream) : launch_gram_d<128, float, 96>(a, G, stream);
    case 128: return bf ? launch_gram_d<128, uint16_t>(a, G, stream) : launch_gram_d<128, float>(a, G, stream);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_boundary(const ForwardArgs& a, int d, const double* G, float* seg_A, hipStream_t stream) {
  switch (d) {
    case 32: return launch_boundary_d<32>(a, G, seg_A, stream);
    case 64: return launch_boundary_d<64>(a, G, seg_A, stream);
    case 96: return launch_boundary_d<128, 96>(a, G, seg_A, stream);
    case 128: return launch_boundary_d<128>(a, G, seg_A, stream);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_combine(const ForwardArgs& a, int d, float* seg_S, hipStream_t stream) {
  switch (d) {
    case 32: return launch_combine_d<32>(a, seg_S, stream);
    case 64: return launch_combine_d<64>(a, seg_S, stream);
    case 96: return launch_combine_d<96>(a, seg_S, stream);
    case 128: return launch_combine_d<128>(a, seg_S, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace vla
