// Internal declarations shared by the HIP translation units of libvla (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vla {

struct ForwardArgs {
  const void* q;
  const void* k;
  const void* v;
  const float* S0;
  const float* A0;
  void* o;
  float* S_T;
  float* A_T;
  int n_heads;  // B*H
  int T;
  float lambda0;
  float eps;
  float* ws;  // device workspace (two-phase mode), else nullptr
  // the remaining lines of Algorithm 1 (general scan and general block kernels)
  const void* u;
  float u_scale;
  int refresh_period;
  float refresh_eta;
  int step_offset;
  int normalise_output;
  int feature_map;
  const float* zkey0;
  float* zkey_T;
  // time segments (time-parallel mode; n_seg == 1 everywhere else)
  int n_seg = 1;                  // segments per head
  int seg_blocks = 0;             // 16-token blocks per segment (the last one may hold fewer)
  const float* seg_A = nullptr;   // [n_heads][n_seg][d][d]  A at the start of every segment
  const float* seg_S = nullptr;   // [n_heads][n_seg][d][d]  S at the start of every segment
  float* seg_PQ = nullptr;        // [n_heads][n_seg][2][d][d]  per-segment affine map of the S recurrence
  const float* seg_zkey = nullptr;  // [n_heads][n_seg][d]  key sum at the start of every segment (normalised read-out)
  // Rows of S (size of the value heads) where a segment kernel takes it at run time; 0: as many as columns.
  // With d_v != d the per-segment arrays hold seg_S [d_v][d] and seg_PQ P [d][d] then Q [d_v][d].
  int d_v = 0;
};

// bf16 <-> f32 helpers on raw bit patterns (bf16 is the upper half of an IEEE float32).
__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t x = __float_as_uint(f);
  if ((x & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((x >> 16) | 0x40u);  // quiet NaN
  x += 0x7fffu + ((x >> 16) & 1u);
  return static_cast<uint16_t>(x >> 16);
}

// Token-by-token scan, one workgroup per head (vla_scan.hip); every pair of head sizes d_k, d_v.
bool scan_supported(int d_k, int d_v);
hipError_t launch_scan(const ForwardArgs& a, int d_k, int d_v, int io_dtype, hipStream_t stream);
// Same, with the optional lines of Algorithm 1 (separate u, refresh, normalised read-out, ELU+1).
hipError_t launch_scan_general(const ForwardArgs& a, int d_k, int d_v, int io_dtype, hipStream_t stream);


// Block form on FP32 MFMA, 16 tokens per block (vla_chunk.hip); head sizes 16, 32, 64, 96 and 128, and value
// heads half or twice as wide as the key heads.
bool chunk_supported(int d);
bool chunk_supported(int d_k, int d_v);
// Head sizes of the two-phase and time-parallel modes.
inline bool block_family_supported(int d) { return d == 32 || d == 64 || d == 96 || d == 128; }
hipError_t launch_chunk(const ForwardArgs& a, int d_k, int d_v, int io_dtype, hipStream_t stream);
// Same block form, several heads per workgroup (vla_chunk_multihead.hip); head sizes 32 and 64.
// launch_chunk picks it by head size and head count (prefer_multihead).
bool prefer_multihead(int d, int n_heads);
hipError_t launch_chunk_multihead(const ForwardArgs& a, int d, int io_dtype, hipStream_t stream);
// Same block form with the optional lines of Algorithm 1 (vla_chunk_general.hip); every head size.
inline bool general_block_supported(int d) { return d == 16 || d == 32 || d == 64 || d == 96 || d == 128; }
hipError_t launch_chunk_general(const ForwardArgs& a, int d, int d_v, int io_dtype, hipStream_t stream);
// Its A chain alone, one workgroup per (head, time segment), writing the workspace records of the two-phase and
// time-parallel modes (head sizes 32, 64, 96, 128).
hipError_t launch_a_scan_general(const ForwardArgs& a, int d, int io_dtype, hipStream_t stream);


// Two-phase split (vla_two_phase.hip): A recurrence first, then the rows of S on many workgroups.
// (d: key heads; the value head size is a.d_v: any supported size)
size_t two_phase_workspace_bytes(int n_heads, int T, int d);
hipError_t launch_two_phase(const ForwardArgs& a, int d, int io_dtype, hipStream_t stream);

// Time-parallel mode: the sequence is cut into segments that run concurrently (vla_two_phase.hip drives it,
// vla_segments.hip holds the kernels that compute the state at the segment boundaries).
struct SegmentPlan {
  int n_seg;       // >= 1
  int seg_blocks;  // 16-token blocks per segment
};
// `general`: the call carries a separate penalty direction or the normalised read-out
SegmentPlan plan_segments(int n_heads, int T, int d, bool general, int requested);
size_t time_parallel_workspace_bytes(int n_heads, int T, int d, int d_v, bool general, int requested_segments);
hipError_t launch_time_parallel(const ForwardArgs& a, int d, int io_dtype, int requested_segments,
                                hipStream_t stream);
// Boundary kernels (vla_segments.hip).  All buffers are device memory inside the caller's workspace.
//   gram:      G[h][s] = sum over the tokens of segments 0..s of u u^T (u = k^ unless the caller supplies
//              penalty directions), float64 [d][d]
//   boundary:  seg_A[h][s] = inverse(inverse(A0[h]) + G[h][s-1]) rounded to float32
//   combine:   seg_S[h][0] = S0[h];  seg_S[h][s+1] = seg_S[h][s] P[h][s] + Q[h][s]  (a.d_v rows)
hipError_t launch_gram(const ForwardArgs& a, int d, int io_dtype, double* G, hipStream_t stream);
hipError_t launch_boundary(const ForwardArgs& a, int d, const double* G, float* seg_A, hipStream_t stream);
hipError_t launch_combine(const ForwardArgs& a, int d, float* seg_S, hipStream_t stream);
//   key sums:  seg_zkey[h][s] = zkey0[h] + sum of the keys (after the feature map) of every token before segment s;
//              `part` [n_heads][n_seg][d] float64 is scratch
hipError_t launch_keysum(const ForwardArgs& a, int d, int io_dtype, double* part, float* seg_zkey,
                         hipStream_t stream);


// One decode step for every head, state updated in place (vla_decode.hip).  `opt` carries eps and the
// optional lines of Algorithm 1 (u, refresh schedule, read-out normaliser, feature map, key sum).  Value heads
// half or twice as wide as the key heads run on the plain kernel only (no options).
bool decode_supported(int d_k, int d_v, bool options);
hipError_t launch_decode(const void* q, const void* k, const void* v, float* S, float* A, void* o,
                         int n_heads, int d_k, int d_v, int io_dtype, const ForwardArgs& opt,
                         hipStream_t stream);

}  // namespace vla
