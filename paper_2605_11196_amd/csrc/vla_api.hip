// Host side of the C ABI declared in include/vla.h: validation, mode selection, dispatch.
#include "../../include/vla.h"

#include "vla_common.h"

#include <stdio.h>

#include <mutex>

// Workspace of vla_forward_static: one array per GPU, part of the library's device image, held until the
// process ends.  In host code the name is only a handle for hipGetSymbolAddress; the kernels get the
// device address that call returns.
constexpr size_t kScratchBytes = size_t{64} << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each GPU, looked up once

// Address of the current device's copy of `scratch` (nullptr and a message on failure).
void* scratch_of_current_device() {
  int dev = -1;
  hipError_t err = hipGetDevice(&dev);
  if (err != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    fprintf(stderr, "libvla: vla_forward_static: no usable current device (%s, device %d)\n",
            hipGetErrorString(err), dev);
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (err != hipSuccess || p == nullptr) {
      fprintf(stderr, "libvla: vla_forward_static: hipGetSymbolAddress failed on device %d: %s\n", dev,
              hipGetErrorString(err));
      return nullptr;
    }
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

constexpr int kVersion = 600;  // 0.6.0

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// A caller buffer as a byte range; `written` marks what the kernels store to.
struct Range {
  const void* p;
  size_t bytes;
  bool written;
};
bool ranges_overlap(const Range& a, const Range& b) {
  if (a.p == nullptr || b.p == nullptr || a.bytes == 0 || b.bytes == 0) return false;
  const uintptr_t a0 = reinterpret_cast<uintptr_t>(a.p), b0 = reinterpret_cast<uintptr_t>(b.p);
  return a0 < b0 + b.bytes && b0 < a0 + a.bytes;
}
// No written buffer may overlap any other buffer of the call, in whole or in part, except for the three exact
// aliases the interface allows (the state and key-sum outputs written over their own inputs).
bool buffers_disjoint(const Range* r, int n, const void* const (*alias)[2], int n_alias) {
  for (int i = 0; i < n; ++i) {
    if (!r[i].written) continue;
    for (int j = 0; j < n; ++j) {
      if (j == i || (r[j].written && j < i)) continue;   // written pairs are looked at once
      if (!ranges_overlap(r[i], r[j])) continue;
      bool allowed = false;
      for (int a = 0; a < n_alias; ++a) {
        allowed = allowed || (r[i].p == r[j].p && r[i].bytes == r[j].bytes &&
                              ((r[i].p == alias[a][0] && r[j].p == alias[a][1]) ||
                               (r[i].p == alias[a][1] && r[j].p == alias[a][0])));
      }
      if (!allowed) return false;
    }
  }
  return true;
}

vla_opts resolve_opts(const vla_opts* o) {
  vla_opts r;
  vla_default_opts(&r);
  if (o != nullptr) r = *o;
  return r;
}

// Shared shape/enum checks; returns VLA_OK when a kernel exists for the request.
int check_shape(int B, int H, int T, int d_k, int d_v, int io_dtype, const vla_opts& o) {
  if (B <= 0 || H <= 0 || T < 0 || d_k <= 0 || d_v <= 0) return VLA_ERR_INVALID_ARG;
  if (io_dtype != VLA_F32 && io_dtype != VLA_BF16) return VLA_ERR_INVALID_ARG;
  if (o.mode < VLA_MODE_AUTO || o.mode > VLA_MODE_TIME_PARALLEL) return VLA_ERR_INVALID_ARG;
  if (o.segments < 0) return VLA_ERR_INVALID_ARG;
  if (!(o.lambda0 > 0.0f) || !(o.eps > 0.0f)) return VLA_ERR_INVALID_ARG;
  if (o.refresh_period < 0 || o.step_offset < 0 || !(o.u_scale == o.u_scale)) return VLA_ERR_INVALID_ARG;
  // step indices (step_offset + t + 1, with a block of look-ahead) are 32-bit in the kernels
  if (static_cast<long long>(o.step_offset) + T + 64 > 0x7fffffffLL) return VLA_ERR_INVALID_ARG;
  if (static_cast<long long>(B) * H > 0x7fffffffLL) return VLA_ERR_INVALID_ARG;
  // kernels address one head's [T, d] slab with 32-bit byte offsets
  if (static_cast<long long>(T) * (d_k > d_v ? d_k : d_v) * 4 >= 0x7fffffffLL) return VLA_ERR_UNSUPPORTED;
  if (!vla::scan_supported(d_k, d_v)) return VLA_ERR_UNSUPPORTED;
  return VLA_OK;
}

// true when an optional line of Algorithm 1 that only the general kernels carry is switched on
bool needs_general_kernel(const vla_opts& o) {
  return o.u != nullptr || o.refresh_period > 0 || o.normalise_output != 0 || o.zkey0 != nullptr ||
         o.zkey_T != nullptr;
}
// true when any of the optional lines of Algorithm 1 is switched on (the plain block kernel carries the
// feature map by itself)
bool general_path(const vla_opts& o) { return needs_general_kernel(o) || o.feature_map != 0; }

// AUTO: options other than the feature map -> the block kernel that carries them; few heads on a long
// sequence -> time-parallel (segments of the sequence run concurrently and the S rows spread over d/16 times
// more workgroups than there are heads); otherwise the fused block kernel.  Every supported shape has a block
// kernel; the scan family is the fallback should one be missing.
int pick_mode(int B, int H, int T, int d, int d_v, const vla_opts& o) {
  if (o.mode != VLA_MODE_AUTO) return o.mode;
  if (!vla::chunk_supported(d, d_v)) return VLA_MODE_SCAN;
  const int with_options = vla::general_block_supported(d) ? VLA_MODE_CHUNKED : VLA_MODE_SCAN;
  // the identity refresh breaks A_t = M_t^{-1}, which the segment boundaries rest on
  if (o.refresh_period > 0) return with_options;
  if (!vla::block_family_supported(d)) {   // d = 16: no segment modes
    return needs_general_kernel(o) ? with_options : VLA_MODE_CHUNKED;
  }
  const long long heads = static_cast<long long>(B) * H;
  // Measured crossovers against the fused block kernel (bf16, one MI355X; time-parallel against block kernel, ms).
  // The segment kernels gain on the block kernel as the sequence grows (their fixed passes amortise):
  //   d = 128:  T = 2048: 64 heads 0.66 / 0.96, 80 heads 1.09 / 0.97;   T = 4096: 96 heads 1.67 / 1.93, 128: 1.99 / 1.93;
  //             T = 8192: 128 heads 3.66 / 3.85, 160: 4.75 / 3.86;      T = 32768: 128 heads 14.2 / 15.4, 160: 18.9 / 15.4
  //   d =  96:  T = 1024: 64 heads 0.33 / 0.41, 96: 0.55 / 0.41;        T = 2048: 64 heads 0.52 / 0.82, 80: 0.83 / 0.82;
  //             T = 4096: 128 heads 1.52 / 1.64, 160: 1.91 / 1.64;      T = 32768: 128 heads 10.5 / 13.1, 160: 13.7 / 13.1
  //   d =  64:  T = 2048: 192 heads 0.51 / 0.63, 256: 0.60 / 0.63, 320: 0.73 / 0.69;   T = 4096: 320 heads 1.33 / 1.38,
  //             384: 1.78 / 1.38;                                       T = 16384: 320 heads 5.13 / 5.48, 384: 7.02 / 5.47
  //   d =  32:  T = 2048: 512 heads 0.51 / 0.57, 640: 0.59 / 0.58;      T = 16384: 512 heads 3.71 / 4.54, 640: 4.59 / 4.56
  const int t_128 = d == 96 ? 4096 : 8192;   // from here 128 heads still gain at d >= 96
  long long few = d >= 96 ? (T >= t_128 ? 128 : (T >= 4096 ? 96 : 64))
                          : (d >= 64 ? (T >= 4096 ? 320 : 192) : 512);
  // Value heads of another size than the key heads: the same thresholds by the key head size, a notch higher
  // where measured (the block kernel shares the row tiles of S out unevenly, the S rows kernel of the segment
  // modes takes them in turn).  T = 4096: d_k = 64, d_v = 128: 384 heads 2.45 / 2.89, 448: 3.05 / 2.88; d_v = 16:
  // 384 heads 1.56 / 1.68;  d_k = 128, d_v = 64: 128 heads 1.50 / 1.62, 160: 1.88 / 1.63; d_v = 16: 128 heads
  // 1.36 / 1.59;  d_k = 32, d_v = 128: 1280 heads 3.25 / 3.58 (T = 1024: 0.83 / 0.90).
  if (d != d_v) {
    if (d == 64 && T >= 4096) few = 384;
    if (d == 128 && T >= 4096) few = 128;
    if (d == 32 && d_v == 128) few = 1280;
  }
  // Short sequences (half the length): 64 heads at d = 64, T = 512: 0.11 against 0.16 ms, 128 heads 0.16 against
  // 0.16; 256 heads at d = 32: 0.12 against 0.14, 512 heads 0.15 against 0.15.  Not at d = 96, whose Gram sums and boundary inverses run in the d = 128 layout (T = 512:
  // 16 heads 0.26 against 0.21).
  const long long few_short = d >= 96 ? 32 : (d >= 64 ? 64 : 256);
  const int t_short = d == 96 ? 1024 : 512;
  const bool take = T >= 1024 ? heads <= few : (T >= t_short && heads <= few_short);
  if (take) return VLA_MODE_TIME_PARALLEL;
  return needs_general_kernel(o) ? with_options : VLA_MODE_CHUNKED;
}

bool mode_available(int mode, int d, int d_v, const vla_opts& o) {
  if (mode == VLA_MODE_SCAN) return true;   // every pair of head sizes, with or without options
  if (!vla::chunk_supported(d, d_v)) return false;
  if (mode == VLA_MODE_CHUNKED) return !needs_general_kernel(o) || vla::general_block_supported(d);
  // the segment modes carry every option but the identity refresh (A at a segment boundary is the explicit
  // inverse of a prefix sum only without it)
  if (mode == VLA_MODE_TWO_PHASE || mode == VLA_MODE_TIME_PARALLEL) {
    return o.refresh_period == 0 && vla::block_family_supported(d);
  }
  return false;
}

// The segment modes launch up to d/8 workgroups per (head, segment) pair and index pairs with 32-bit integers
// (at most 256 segments per head).
bool segment_grid_fits(int mode, long long heads, int d) {
  if (mode != VLA_MODE_TWO_PHASE && mode != VLA_MODE_TIME_PARALLEL) return true;
  return heads * 256 * (d / 8) <= 0x7fffffffLL;
}

}  // namespace

extern "C" {

void vla_default_opts(vla_opts* opts) {
  if (opts == nullptr) return;
  opts->lambda0 = 0.1f;
  opts->eps = 1e-4f;
  opts->mode = VLA_MODE_AUTO;
  opts->u = nullptr;
  opts->u_scale = 1.0f;
  opts->refresh_period = 0;
  opts->refresh_eta = 1e-3f;
  opts->step_offset = 0;
  opts->normalise_output = 0;
  opts->feature_map = 0;
  opts->zkey0 = nullptr;
  opts->zkey_T = nullptr;
  opts->segments = 0;
}

int vla_version(void) { return kVersion; }

const char* vla_status_string(int status) {
  switch (status) {
    case VLA_OK: return "VLA_OK";
    case VLA_ERR_INVALID_ARG: return "VLA_ERR_INVALID_ARG";
    case VLA_ERR_UNSUPPORTED: return "VLA_ERR_UNSUPPORTED";
    case VLA_ERR_WORKSPACE: return "VLA_ERR_WORKSPACE";
    case VLA_ERR_HIP: return "VLA_ERR_HIP";
    default: return "VLA_ERR_UNKNOWN";
  }
}

int vla_resolve_mode(int B, int H, int T, int d_k, int d_v, int io_dtype, const vla_opts* opts) {
  const vla_opts o = resolve_opts(opts);
  if (check_shape(B, H, T, d_k, d_v, io_dtype, o) != VLA_OK) return -1;
  const int mode = pick_mode(B, H, T, d_k, d_v, o);
  if (!segment_grid_fits(mode, static_cast<long long>(B) * H, d_k)) return -1;
  return mode_available(mode, d_k, d_v, o) ? mode : -1;
}

size_t vla_forward_workspace_bytes(int B, int H, int T, int d_k, int d_v, int io_dtype,
                                   const vla_opts* opts) {
  const vla_opts o = resolve_opts(opts);
  if (check_shape(B, H, T, d_k, d_v, io_dtype, o) != VLA_OK) return 0;
  const int mode = pick_mode(B, H, T, d_k, d_v, o);
  if (!mode_available(mode, d_k, d_v, o)) return 0;
  if (!segment_grid_fits(mode, static_cast<long long>(B) * H, d_k)) return 0;
  if (mode == VLA_MODE_TWO_PHASE) return vla::two_phase_workspace_bytes(B * H, T, d_k);
  if (mode == VLA_MODE_TIME_PARALLEL) {
    return vla::time_parallel_workspace_bytes(B * H, T, d_k, d_v, needs_general_kernel(o), o.segments);
  }
  return 0;
}

}  // extern "C"

namespace {

// vla_forward and vla_forward_static.  `own_scratch`: the workspace is the library's static array, looked up
// only once the request is known to be valid and to need one.
int forward_impl(const void* q, const void* k, const void* v, const float* S0, const float* A0,
                 void* o, float* S_T, float* A_T, int B, int H, int T, int d_k, int d_v,
                 int io_dtype, const vla_opts* opts, void* workspace, size_t workspace_bytes,
                 bool own_scratch, void* stream) {
  const vla_opts op = resolve_opts(opts);
  const int st = check_shape(B, H, T, d_k, d_v, io_dtype, op);
  if (st != VLA_OK) return st;
  if (T > 0 && (q == nullptr || k == nullptr || v == nullptr || o == nullptr)) {
    return VLA_ERR_INVALID_ARG;
  }
  const void* ptrs[] = {q, k, v, S0, A0, o, S_T, A_T, workspace, op.u, op.zkey0, op.zkey_T};
  for (const void* p : ptrs) {
    if (p != nullptr && !aligned16(p)) return VLA_ERR_INVALID_ARG;
  }
  {
    const size_t es = io_dtype == VLA_BF16 ? 2 : 4;
    const size_t heads = static_cast<size_t>(B) * H;
    const size_t nk = heads * T * d_k * es, nv = heads * T * d_v * es;
    const size_t nS = heads * d_v * d_k * 4, nA = heads * d_k * d_k * 4, nz = heads * d_k * 4;
    const Range r[] = {{q, nk, false},        {k, nk, false},         {v, nv, false},  {op.u, nk, false},
                       {S0, nS, false},       {A0, nA, false},        {op.zkey0, nz, false},
                       {o, nv, true},         {S_T, nS, true},        {A_T, nA, true}, {op.zkey_T, nz, true},
                       {workspace, workspace_bytes, true}};
    const void* const alias[][2] = {{S_T, S0}, {A_T, A0}, {op.zkey_T, op.zkey0}};
    if (!buffers_disjoint(r, 12, alias, 3)) return VLA_ERR_INVALID_ARG;
  }

  int mode = pick_mode(B, H, T, d_k, d_v, op);
  if (!mode_available(mode, d_k, d_v, op)) return VLA_ERR_UNSUPPORTED;
  if (!segment_grid_fits(mode, static_cast<long long>(B) * H, d_k)) return VLA_ERR_UNSUPPORTED;
  const size_t need = vla_forward_workspace_bytes(B, H, T, d_k, d_v, io_dtype, &op);
  if (own_scratch && need > 0 && need <= kScratchBytes) {
    workspace = scratch_of_current_device();
    if (workspace == nullptr) return VLA_ERR_HIP;
    workspace_bytes = kScratchBytes;
  }
  if (need > 0 && (workspace == nullptr || workspace_bytes < need)) {
    // AUTO never fails for want of a workspace: it falls back to the fused block kernel
    if (op.mode != VLA_MODE_AUTO) {
      if (own_scratch) {
        fprintf(stderr, "libvla: vla_forward_static: this call needs %zu bytes of workspace, the static "
                        "array holds %zu; use vla_forward with a workspace of the caller's\n",
                need, kScratchBytes);
      }
      return VLA_ERR_WORKSPACE;
    }
    mode = VLA_MODE_CHUNKED;
  }
  if (T == 0 && S_T == nullptr && A_T == nullptr && op.zkey_T == nullptr) return VLA_OK;  // nothing to do

  vla::ForwardArgs a;
  a.q = q; a.k = k; a.v = v; a.S0 = S0; a.A0 = A0;
  a.o = o; a.S_T = S_T; a.A_T = A_T;
  a.n_heads = B * H;
  a.T = T;
  a.lambda0 = op.lambda0;
  a.eps = op.eps;
  a.ws = static_cast<float*>(workspace);
  a.u = op.u; a.u_scale = op.u_scale;
  a.refresh_period = op.refresh_period; a.refresh_eta = op.refresh_eta; a.step_offset = op.step_offset;
  a.normalise_output = op.normalise_output; a.feature_map = op.feature_map;
  a.zkey0 = op.zkey0; a.zkey_T = op.zkey_T;
  a.d_v = d_v;

  hipError_t err = hipSuccess;
  switch (mode) {
    case VLA_MODE_SCAN:
      err = general_path(op)
                ? vla::launch_scan_general(a, d_k, d_v, io_dtype, static_cast<hipStream_t>(stream))
                : vla::launch_scan(a, d_k, d_v, io_dtype, static_cast<hipStream_t>(stream));
      break;
    case VLA_MODE_CHUNKED:
      err = needs_general_kernel(op)
                ? vla::launch_chunk_general(a, d_k, d_v, io_dtype, static_cast<hipStream_t>(stream))
                : vla::launch_chunk(a, d_k, d_v, io_dtype, static_cast<hipStream_t>(stream));
      break;
    case VLA_MODE_TWO_PHASE:
      err = vla::launch_two_phase(a, d_k, io_dtype, static_cast<hipStream_t>(stream));
      break;
    case VLA_MODE_TIME_PARALLEL:
      err = vla::launch_time_parallel(a, d_k, io_dtype, op.segments, static_cast<hipStream_t>(stream));
      break;
    default:
      return VLA_ERR_UNSUPPORTED;
  }
  if (err != hipSuccess) {
    fprintf(stderr, "libvla: kernel launch failed: %s (%d)\n", hipGetErrorString(err),
            static_cast<int>(err));
    return VLA_ERR_HIP;
  }
  return VLA_OK;
}

}  // namespace

extern "C" {

int vla_forward(const void* q, const void* k, const void* v, const float* S0, const float* A0,
                void* o, float* S_T, float* A_T, int B, int H, int T, int d_k, int d_v,
                int io_dtype, const vla_opts* opts, void* workspace, size_t workspace_bytes,
                void* stream) {
  return forward_impl(q, k, v, S0, A0, o, S_T, A_T, B, H, T, d_k, d_v, io_dtype, opts, workspace,
                      workspace_bytes, false, stream);
}

int vla_forward_static(const void* q, const void* k, const void* v, const float* S0, const float* A0,
                       void* o, float* S_T, float* A_T, int B, int H, int T, int d_k, int d_v,
                       int io_dtype, const vla_opts* opts, void* stream) {
  return forward_impl(q, k, v, S0, A0, o, S_T, A_T, B, H, T, d_k, d_v, io_dtype, opts, nullptr, 0, true,
                      stream);
}

int vla_decode_step(const void* q, const void* k, const void* v, float* S, float* A, void* o, int B,
                    int H, int d_k, int d_v, int io_dtype, const vla_opts* opts, void* stream) {
  const vla_opts op = resolve_opts(opts);
  const int st = check_shape(B, H, 1, d_k, d_v, io_dtype, op);
  if (st != VLA_OK) return st;
  if (!vla::decode_supported(d_k, d_v, general_path(op))) return VLA_ERR_UNSUPPORTED;
  if (q == nullptr || k == nullptr || v == nullptr || S == nullptr || A == nullptr || o == nullptr) {
    return VLA_ERR_INVALID_ARG;
  }
  const void* ptrs[] = {q, k, v, S, A, o, op.u, op.zkey0, op.zkey_T};
  for (const void* p : ptrs) {
    if (p != nullptr && !aligned16(p)) return VLA_ERR_INVALID_ARG;
  }
  {
    const size_t es = io_dtype == VLA_BF16 ? 2 : 4;
    const size_t heads = static_cast<size_t>(B) * H;
    const size_t nk = heads * d_k * es, nv = heads * d_v * es, nz = heads * d_k * 4;
    const Range r[] = {{q, nk, false},          {k, nk, false}, {v, nv, false}, {op.u, nk, false},
                       {op.zkey0, nz, false},   {o, nv, true},  {S, heads * d_v * d_k * 4, true},
                       {A, heads * d_k * d_k * 4, true},        {op.zkey_T, nz, true}};
    const void* const alias[][2] = {{op.zkey_T, op.zkey0}};
    if (!buffers_disjoint(r, 9, alias, 1)) return VLA_ERR_INVALID_ARG;
  }
  vla::ForwardArgs fa{};
  fa.eps = op.eps;
  fa.u = op.u; fa.u_scale = op.u_scale;
  fa.refresh_period = op.refresh_period; fa.refresh_eta = op.refresh_eta; fa.step_offset = op.step_offset;
  fa.normalise_output = op.normalise_output; fa.feature_map = op.feature_map;
  fa.zkey0 = op.zkey0; fa.zkey_T = op.zkey_T;
  const hipError_t err = vla::launch_decode(q, k, v, S, A, o, B * H, d_k, d_v, io_dtype, fa,
                                            static_cast<hipStream_t>(stream));
  if (err != hipSuccess) {
    fprintf(stderr, "libvla: kernel launch failed: %s (%d)\n", hipGetErrorString(err),
            static_cast<int>(err));
    return VLA_ERR_HIP;
  }
  return VLA_OK;
}

}  // extern "C"
