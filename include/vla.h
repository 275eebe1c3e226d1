/*
 * vla.h -- C ABI of the MI355X (gfx950) Variational Linear Attention forward library.
 *
 * One operation: the causal per-head VLA forward recurrence (paper Section 3.3,
 * eq. (sm), eq. (s-update), numerator of eq. (output); Algorithm 1).  For every
 * (batch b, head h) independently, starting from S = S0[b,h], A = A0[b,h], for
 * t = 1..T:
 *
 *     k^_t     = k_t / max(||k_t||, eps)                       (Section 3.1)
 *     u_t      = k^_t               (penalty direction aligned with the key, Section 7.1)
 *     z_t      = A_{t-1} u_t ;  delta_t = max(1 + u_t . z_t, eps)
 *     A_t      = A_{t-1} - z_t z_t^T / delta_t                 (eq. (sm))
 *     alpha^_t = A_t k^_t / max(||A_t k^_t||, eps)             (post-update A)
 *     e_t      = v_t - S_{t-1} k^_t
 *     S_t      = S_{t-1} + e_t alpha^_t^T                      (eq. (s-update))
 *     o_t      = S_t q_t                                       (post-update S)
 *
 * and finally S_T, A_T are written out.  The other lines of Algorithm 1 (a separate
 * penalty direction u, the periodic identity refresh, the denominator of eq. (output)
 * and the ELU+1 feature map) are off by default and switched on through vla_opts.
 *
 * Every pointer is a DEVICE pointer unless stated otherwise.  The library never
 * allocates, frees or retains memory: the caller owns every buffer for the
 * duration of the call's execution on `stream`.  Calls are asynchronous with
 * respect to the host (kernels are enqueued on `stream`, no host synchronisation)
 * and re-entrant.  All validation happens on the host before anything is enqueued: with
 * VLA_ERR_INVALID_ARG, VLA_ERR_UNSUPPORTED or VLA_ERR_WORKSPACE nothing has been launched and no
 * output has been touched.  VLA_ERR_HIP reports a launch the HIP runtime refused; in the modes
 * that run several kernels back to back, earlier kernels of the call may already be enqueued
 * then and the outputs and the workspace hold unspecified values.
 */
#ifndef VLA_H_
#define VLA_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Element type of q, k, v and o.  The states S and A are always float32, and all
 * arithmetic is float32 regardless of the I/O type (bf16 inputs are widened
 * exactly; o is rounded to nearest-even on the final store). */
typedef enum { VLA_F32 = 0, VLA_BF16 = 1 } vla_dtype;

/* Which kernel family runs the recurrence.
 *   AUTO     : the library picks: CHUNKED when the identity refresh is switched on or the shape has no
 *              segment kernels; else TIME_PARALLEL for few heads (d = 128 and 96: B*H <= 64, 96 from
 *              T = 4096, 128 from T = 8192 (from 4096 at d = 96); d = 64: 192, 320 from T = 4096;
 *              d = 32: 512) and T >= 1024, or from T = 512 for B*H <= 32, 64, 256 heads at d = 128, 64,
 *              32 (d_k != d_v: by d_k, with 384 heads at d_k = 64 and 128 at d_k = 128 from T = 4096,
 *              1280 at d_k = 32 with d_v = 128), if the caller passed the workspace
 *              vla_forward_workspace_bytes() asks for (else CHUNKED); CHUNKED otherwise.
 *   SCAN     : one workgroup per (b,h) walks the tokens one by one with A and S
 *              resident in registers (FP32 vector ALU).
 *   CHUNKED  : tokens are processed in blocks; the block form of the same
 *              recurrence turns the matrix-vector work into dense FP32 matrix
 *              products (MFMA).  Same result up to float32 rounding order.  A second block kernel
 *              carries the options of Algorithm 1.
 *   TWO_PHASE: phase 1 runs the A recurrence and writes k^_t, alpha^_t to the
 *              workspace; phase 2 runs the S recurrence with the rows of S spread
 *              over several workgroups (for small B*H).  Allowed because A never
 *              reads S (eq. (sm)); Algorithm 2 takes k^, alpha^ as given inputs.
 *   TIME_PARALLEL: TWO_PHASE with the sequence cut into segments that run concurrently (for small
 *              B*H and long T).  Without the refresh, A at a segment boundary is the explicit
 *              inverse (A_0^{-1} + sum of u u^T up to there)^{-1} of Section 3.2 / eq. (penalty) (u = k^
 *              unless opts->u is given), computed in float64 from one Gram matrix per segment; S at a
 *              boundary follows by composing the per-segment affine maps S -> S P + Q of
 *              eq. (s-update); the key sum of the normalised read-out at a boundary is a prefix sum.
 *              Inside a segment the recurrence is the same exact block form.  Same result up to float32
 *              rounding.
 */
typedef enum {
  VLA_MODE_AUTO = 0,
  VLA_MODE_SCAN = 1,
  VLA_MODE_CHUNKED = 2,
  VLA_MODE_TWO_PHASE = 3,
  VLA_MODE_TIME_PARALLEL = 4
} vla_mode;

typedef enum {
  VLA_OK = 0,
  VLA_ERR_INVALID_ARG = 1, /* null required pointer, non-positive size, misaligned pointer, bad enum */
  VLA_ERR_UNSUPPORTED = 2, /* valid request this build has no kernel for (head sizes, mode, option) */
  VLA_ERR_WORKSPACE = 3,   /* workspace missing or smaller than vla_forward_workspace_bytes() */
  VLA_ERR_HIP = 4          /* the HIP runtime reported an error at launch */
} vla_status;

/* Options; pass NULL for the defaults in brackets.  Always initialise the struct with
 * vla_default_opts() and then change fields: later library versions may append fields.
 *
 * The fields after `mode` switch on the remaining lines of Algorithm 1 (paper, pseudocode appendix).
 * SCAN and CHUNKED carry all of them; TWO_PHASE and TIME_PARALLEL carry all but the identity refresh
 * (asking for them with refresh_period > 0 returns VLA_ERR_UNSUPPORTED, and AUTO then selects CHUNKED): with
 * the refresh A_t is no longer the inverse of a prefix sum, which the segment boundaries rest on.
 * feature_map on its own changes no routing. */
typedef struct vla_opts {
  float lambda0; /* [0.1]  A_0 = I / lambda0, used only when A0 == NULL (Section 3.2) */
  float eps;     /* [1e-4] floor of every denominator: ||k||, delta, ||A k^||, ||u|| and the
                    read-out denominator (Section 5.4) */
  int mode;      /* [VLA_MODE_AUTO] a vla_mode */
  const void* u; /* [NULL] device, [B, H, T, d_k], io_dtype: raw penalty directions u~_t of
                    eq. (penalty); the recurrence uses u_t = u_scale * u~_t / max(||u~_t||, eps).
                    NULL: u_t = k^_t (Section 7.1) */
  float u_scale; /* [1.0]  1/sqrt(d_h) reproduces the scaling in Algorithm 1 */
  int refresh_period;   /* [0 = off] > 0: A += refresh_eta * I after the rank-1 update (and before the
                           write direction is formed) at every step whose 1-based index
                           step_offset + t is a multiple of refresh_period (Algorithm 1 uses 20) */
  float refresh_eta;    /* [1e-3] */
  int step_offset;      /* [0] tokens already processed by earlier calls of a split sequence; only
                           the refresh schedule depends on it */
  int normalise_output; /* [0] 1: o_t = S_t q_t / max(q_t . zkey_t, eps) with the running key sum
                           zkey_t = zkey_0 + sum_{s<=t} k_s of eq. (output); k_s is the key as used
                           (after feature_map, before L2 normalisation) */
  int feature_map;      /* [0] 1: q and k are replaced by ELU(x) + 1 elementwise on load (Section 3.3) */
  const float* zkey0;   /* [NULL = 0] device, [B, H, d_k] float32: key sum carried in from earlier calls */
  float* zkey_T;        /* [NULL = not wanted] device, [B, H, d_k] float32: key sum after the last token;
                           may alias zkey0 */
  int segments;         /* [0 = the library chooses] TIME_PARALLEL only: number of time segments (at most
                           256; capped at one per 16 tokens).  Sizes the workspace, so pass the same
                           value to vla_forward_workspace_bytes() and vla_forward() */
} vla_opts;

/* Fills *opts with the defaults above. */
void vla_default_opts(vla_opts* opts);

/* Bytes of device workspace vla_forward needs for these arguments (0 for the
 * modes that need none).  Returns 0 as well when the arguments are invalid --
 * vla_forward will then report the error.  Pass the options of the call itself: with `segments` left at 0
 * the number of segments, and so the size, also depends on whether u, normalise_output or the zkey
 * pointers are set (a workspace sized for other options may be refused with VLA_ERR_WORKSPACE). */
size_t vla_forward_workspace_bytes(int B, int H, int T, int d_k, int d_v, int io_dtype,
                                   const vla_opts* opts);

/*
 * vla_forward -- run the recurrence above for all B*H heads over T tokens.
 *
 *   q, k   [B, H, T, d_k]   io_dtype, contiguous, read-only
 *   v      [B, H, T, d_v]   io_dtype, contiguous, read-only
 *   S0     [B, H, d_v, d_k] float32 row-major, or NULL for S_0 = 0     (Algorithm 1)
 *   A0     [B, H, d_k, d_k] float32 row-major, or NULL for I / lambda0 (Algorithm 1).
 *          Must be symmetric positive definite (precondition, not checked).
 *   o      [B, H, T, d_v]   io_dtype, written
 *   S_T    [B, H, d_v, d_k] float32, written; NULL if not wanted; may be S0 itself
 *   A_T    [B, H, d_k, d_k] float32, written; NULL if not wanted; may be A0 itself
 *          No written buffer (o, S_T, A_T, opts->zkey_T, the workspace) may overlap another buffer of
 *          the call, in whole or in part -- the byte ranges are compared on the host and an overlap
 *          returns VLA_ERR_INVALID_ARG -- with three exceptions: S_T == S0, A_T == A0 and
 *          zkey_T == zkey0 (the same pointer: the state is then updated in place).
 *   B, H   >= 1;  T >= 0 (T == 0 copies the initial state to S_T / A_T)
 *   d_k, d_v in {16, 32, 64, 96, 128}, any pair (S is d_v x d_k).  SCAN and CHUNKED for every pair and
 *          every option (with d_k != d_v the waves of a head share out the d_v / 16 row tiles of S);
 *          TWO_PHASE and TIME_PARALLEL for d_k >= 32 with any d_v (every option but the identity
 *          refresh); AUTO routes by d_k as above
 *   opts   host pointer or NULL
 *   workspace, workspace_bytes: device scratch of at least
 *          vla_forward_workspace_bytes(...) bytes (may be NULL/0 when that is 0)
 *   stream a hipStream_t passed as void*; NULL is the default stream
 *
 * All device pointers must be 16-byte aligned.  Returns a vla_status.
 * Running [0,T1) and then [T1,T) with the carried S_T, A_T gives the same result
 * as one call over [0,T) (the fixed-size state is the whole memory, Section 7.4).
 */
int vla_forward(const void* q, const void* k, const void* v, const float* S0, const float* A0,
                void* o, float* S_T, float* A_T, int B, int H, int T, int d_k, int d_v,
                int io_dtype, const vla_opts* opts, void* workspace, size_t workspace_bytes,
                void* stream);

/*
 * vla_forward_static -- vla_forward for callers that cannot allocate device memory or have none to pass as a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and same results as vla_forward, without the workspace pair: the modes that need
 * a workspace (TWO_PHASE, TIME_PARALLEL, and AUTO where it resolves to them) use an array of
 * 64 MiB (67,108,864 bytes) that is part of the library's device image -- every GPU the library runs on holds
 * its own copy from the first use of the library on it until the process ends.  The call allocates and frees
 * nothing.
 *
 *   - A request whose vla_forward_workspace_bytes() exceeds 64 MiB returns VLA_ERR_WORKSPACE (with a
 *     message on stderr) when TWO_PHASE or TIME_PARALLEL was asked for by name; AUTO runs CHUNKED instead,
 *     as vla_forward does when it is given no workspace.
 *   - The device that owns the buffers and `stream` must be the current device.  The first call on a device
 *     looks the array's address up once (hipGetSymbolAddress; VLA_ERR_HIP if that fails): make that call
 *     before a stream capture begins.
 *   - All calls on one GPU share that GPU's array: two calls that need it and may overlap in time (different
 *     streams, or graphs replayed concurrently) race on it.  Calls on one stream are ordered and safe.
 *     Nothing in the array has to start at zero and nothing is kept in it between calls.
 */
int vla_forward_static(const void* q, const void* k, const void* v, const float* S0, const float* A0,
                       void* o, float* S_T, float* A_T, int B, int H, int T, int d_k, int d_v,
                       int io_dtype, const vla_opts* opts, void* stream);

/*
 * vla_decode_step -- one token of the same recurrence for every head, on a state that stays where it is
 * (generation: Section 7.4, the fixed-size state S, A is the whole memory).  Equivalent to vla_forward with
 * T = 1, S0 = S_T = S and A0 = A_T = A, but organised for the memory traffic that dominates a single step
 * (2 d^2 floats of state read and written per head against 10 d^2 flop).
 *
 *   q, k   [B, H, d_k]      io_dtype, contiguous, read-only
 *   v      [B, H, d_v]      io_dtype, contiguous, read-only
 *   S      [B, H, d_v, d_k] float32 row-major, updated in place (required)
 *   A      [B, H, d_k, d_k] float32 row-major, updated in place (required; symmetric positive definite)
 *   o      [B, H, d_v]      io_dtype, written; must not overlap any input
 *   d_k, d_v in {16, 32, 64, 96, 128}, any pair, with or without the optional lines of Algorithm 1
 *   opts   host pointer or NULL.  eps and the optional lines of Algorithm 1 are honoured as in vla_forward
 *          with T = 1: u [B, H, d_k] (io_dtype) with u_scale, the identity refresh (this call is step
 *          step_offset + 1 of the schedule), normalise_output with zkey0 / zkey_T [B, H, d_k] (may alias),
 *          feature_map.  lambda0, mode and segments are not used.
 *   stream a hipStream_t passed as void*; NULL is the default stream
 *
 * All device pointers must be 16-byte aligned.  Asynchronous, allocates nothing.  Returns a vla_status.
 */
int vla_decode_step(const void* q, const void* k, const void* v, float* S, float* A, void* o, int B,
                    int H, int d_k, int d_v, int io_dtype, const vla_opts* opts, void* stream);

/* Human-readable name of a vla_status (static storage, never NULL). */
const char* vla_status_string(int status);

/* Library version: major*10000 + minor*100 + patch. */
int vla_version(void);

/* Which concrete mode AUTO resolves to for these arguments when the workspace asked for by
 * vla_forward_workspace_bytes() is passed (a vla_mode, never AUTO), or -1 if the arguments are
 * invalid/unsupported.  Host-only, launches nothing. */
int vla_resolve_mode(int B, int H, int T, int d_k, int d_v, int io_dtype, const vla_opts* opts);

#ifdef __cplusplus
}
#endif
#endif /* VLA_H_ */
