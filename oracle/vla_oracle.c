/*
 * vla_oracle.c -- plain fp64 CPU oracle for the Variational Linear Attention
 * (VLA) causal per-head forward recurrence.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct
 * definition that the GPU library is checked against.  It shares no code,
 * header, table or helper with the HIP path and must never be called from
 * the product path: only the test-suite, the smoke check and the benchmark's
 * "cpu_baseline" leg may load it.
 *
 * What it computes (paper Section 3.3, eq. (sm), eq. (s-update), eq. (output)
 * numerator; Algorithm 1 in the pseudocode appendix), for every (batch, head)
 * independently and for t = 1..T in order:
 *
 *   k^_t   = k_t / max(||k_t||, eps)                     (Section 3.1)
 *   u_t    = k^_t                       (special case u_s = k^_s, Section 7.1)
 *            or  u_scale * u~_t / max(||u~_t||, eps)  for a supplied u~
 *                                                        (eq. (penalty))
 *   z_t    = A_{t-1} u_t
 *   delta  = max(1 + u_t . z_t, eps)
 *   A_t    = A_{t-1} - z_t z_t^T / delta                 (eq. (sm))
 *   a_t    = A_t k^_t            (POST-update A, Appendix A "Why post-update")
 *   alpha^ = a_t / max(||a_t||, eps)
 *   e_t    = v_t - S_{t-1} k^_t                          (PRE-update S)
 *   S_t    = S_{t-1} + e_t alpha^_t^T                    (eq. (s-update))
 *   o_t    = S_t q_t                                     (POST-update S)
 *
 * No algebraic shortcut, blocking, fusion or reordering is applied: every
 * matrix-vector product and rank-1 update is a plain double loop over the
 * full matrix, in the order listed above.
 *
 * Readings taken where the paper is silent or inconsistent:
 *   - the clamp is x / max(||x||, eps), not x / (||x|| + eps); the paper only
 *     says eps = 1e-4 is used "for all denominators" (Section 5.4) and writes
 *     the max() form out for delta (Algorithm 1) and the output denominator.
 *   - by default the identity refresh of Algorithm 1 is off (it would break
 *     A_t = M_t^{-1}), the denominator of eq. (output) is not applied and no
 *     feature map is applied; each of these lines of Algorithm 1 can be
 *     switched on through vla_oracle_opts (refresh after the rank-1 update and
 *     before alpha; phi(x) = ELU(x)+1 on q and k before everything else; the
 *     accumulator of eq. (output) sums the keys as used, before L2 normalisation).
 *   - S is d_v x d_k and o = S q as in eq. (s-update)/(output).
 *
 * Layouts: q,k,u [B,H,T,d_k]; v,o [B,H,T,d_v]; S [B,H,d_v,d_k] row-major;
 * A [B,H,d_k,d_k] row-major.  All host pointers, all double.
 *
 * Pins (tests/test_oracle_pins.py): explicit inverse of M_T; symmetry /
 * positive-definiteness / delta >= 1; ||A_0||_F = sqrt(d)/lambda0 (the
 * paper's printed ~56 at d_h=32, lambda0=0.1); finite-difference Jacobian
 * I - alpha^ k^T structure; orthonormal-key exact recall (Prop. 3);
 * two-key write direction; normalised delta rule when u = 0; Prop. 1
 * inequality; zero-key no-op; state carry; invariances.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#include <stddef.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define VLA_ORACLE_TRACE_WIDTH 8

typedef struct {
  double lambda0;   /* A_0 = I / lambda0 when A0 == NULL (paper: 0.1) */
  double eps;       /* stability floor (paper: 1e-4) */
  const double* u;  /* optional raw penalty directions [B,H,T,d_k]; NULL => u_t = k^_t */
  double u_scale;   /* multiplies a supplied, unit-normalised u (1.0 = eq. (penalty)) */
  /* The remaining switches reproduce the other lines of Algorithm 1; all default to off. */
  int refresh_period;      /* > 0: A += refresh_eta * I after the rank-1 update of every step t (1-based)
                              with t mod period == 0 */
  double refresh_eta;
  int step_offset;         /* tokens processed by earlier calls (only shifts the refresh schedule) */
  int normalise_output;    /* 1: o_t = S_t q_t / max(q_t . zkey_t, eps), zkey_t = zkey_0 + sum_{s<=t} k_s
                              (eq. (output); k_s is the key as used, i.e. after the feature map) */
  int feature_map;         /* 1: q and k are replaced by ELU(x) + 1 elementwise before anything else */
  const double* zkey0;     /* [B,H,d_k] initial key accumulator, NULL => 0 */
  double* zkey_T;          /* [B,H,d_k] final key accumulator, NULL => not wanted */
} vla_oracle_opts;

/* Per-step diagnostics written to trace[((b*H+h)*T + t)*8 + i]:
 *   0: ||S_t||_F   1: ||A_t||_F   2: delta_t (after the clamp)
 *   3: ||e_t||     4: c_t = k^_t . alpha^_t
 *   5: ||k^_t||    6: ||alpha^_t||   7: 1 + u.z before the clamp           */

static double dot(const double* a, const double* b, int n) {
  double s = 0.0;
  for (int i = 0; i < n; ++i) s += a[i] * b[i];
  return s;
}

static double frob(const double* m, size_t n) {
  double s = 0.0;
  for (size_t i = 0; i < n; ++i) s += m[i] * m[i];
  return sqrt(s);
}

/* y = M x, M is rows x cols row-major */
static void matvec(const double* M, const double* x, double* y, int rows, int cols) {
  for (int i = 0; i < rows; ++i) y[i] = dot(M + (size_t)i * cols, x, cols);
}

static void one_head(const double* q, const double* k, const double* v, const double* u_raw,
                     const double* S0, const double* A0, double* o, double* S_T, double* A_T,
                     double* trace, int T, int dk, int dv, double lambda0, double eps,
                     double u_scale, int refresh_period, double refresh_eta, int step_offset, int normalise_output,
                     int feature_map, const double* zkey0, double* zkey_T) {
  double* S = (double*)malloc(sizeof(double) * (size_t)dv * dk);
  double* A = (double*)malloc(sizeof(double) * (size_t)dk * dk);
  double* kh = (double*)malloc(sizeof(double) * dk);
  double* u = (double*)malloc(sizeof(double) * dk);
  double* z = (double*)malloc(sizeof(double) * dk);
  double* a = (double*)malloc(sizeof(double) * dk);
  double* e = (double*)malloc(sizeof(double) * dv);
  double* kf = (double*)malloc(sizeof(double) * dk);   /* key after the feature map */
  double* qf = (double*)malloc(sizeof(double) * dk);   /* query after the feature map */
  double* zkey = (double*)calloc(dk, sizeof(double));  /* running key accumulator (eq. (output)) */
  if (zkey0) memcpy(zkey, zkey0, sizeof(double) * dk);

  if (S0) memcpy(S, S0, sizeof(double) * (size_t)dv * dk);
  else memset(S, 0, sizeof(double) * (size_t)dv * dk);           /* S_0 = 0 (Algorithm 1) */
  if (A0) memcpy(A, A0, sizeof(double) * (size_t)dk * dk);
  else {
    memset(A, 0, sizeof(double) * (size_t)dk * dk);              /* A_0 = I / lambda0 */
    for (int i = 0; i < dk; ++i) A[(size_t)i * dk + i] = 1.0 / lambda0;
  }

  for (int t = 0; t < T; ++t) {
    const double* kt = kf;
    const double* qt = qf;
    const double* vt = v + (size_t)t * dv;

    /* feature map phi(x) = ELU(x) + 1 (Section 3.3): x + 1 for x > 0, exp(x) otherwise */
    for (int j = 0; j < dk; ++j) {
      double kr = k[(size_t)t * dk + j], qr = q[(size_t)t * dk + j];
      kf[j] = feature_map ? (kr > 0.0 ? kr + 1.0 : exp(kr)) : kr;
      qf[j] = feature_map ? (qr > 0.0 ? qr + 1.0 : exp(qr)) : qr;
    }

    /* key normalisation */
    double kn = sqrt(dot(kt, kt, dk));
    double kden = kn > eps ? kn : eps;
    for (int j = 0; j < dk; ++j) kh[j] = kt[j] / kden;

    /* penalty direction */
    if (u_raw) {
      const double* ut = u_raw + (size_t)t * dk;
      double un = sqrt(dot(ut, ut, dk));
      double uden = un > eps ? un : eps;
      for (int j = 0; j < dk; ++j) u[j] = u_scale * (ut[j] / uden);
    } else {
      for (int j = 0; j < dk; ++j) u[j] = kh[j];
    }

    /* Sherman-Morrison: z = A u, delta = 1 + u.z, A -= z z^T / delta */
    matvec(A, u, z, dk, dk);
    double delta_raw = 1.0 + dot(u, z, dk);
    double delta = delta_raw > eps ? delta_raw : eps;
    for (int i = 0; i < dk; ++i)
      for (int j = 0; j < dk; ++j) A[(size_t)i * dk + j] -= z[i] * z[j] / delta;

    /* periodic identity refresh (Algorithm 1), steps counted from 1 */
    if (refresh_period > 0 && (step_offset + t + 1) % refresh_period == 0)
      for (int i = 0; i < dk; ++i) A[(size_t)i * dk + i] += refresh_eta;

    /* write direction from the post-update A */
    matvec(A, kh, a, dk, dk);
    double an = sqrt(dot(a, a, dk));
    double aden = an > eps ? an : eps;
    for (int j = 0; j < dk; ++j) a[j] = a[j] / aden;              /* a now holds alpha^ */

    /* residual against the pre-update S, then the rank-1 write */
    for (int i = 0; i < dv; ++i) e[i] = vt[i] - dot(S + (size_t)i * dk, kh, dk);
    for (int i = 0; i < dv; ++i)
      for (int j = 0; j < dk; ++j) S[(size_t)i * dk + j] += e[i] * a[j];

    /* read-out from the post-update S */
    matvec(S, qt, o + (size_t)t * dv, dv, dk);
    for (int j = 0; j < dk; ++j) zkey[j] += kt[j];
    if (normalise_output) {
      double den = dot(zkey, qt, dk);
      den = den > eps ? den : eps;
      for (int i = 0; i < dv; ++i) o[(size_t)t * dv + i] /= den;
    }

    if (trace) {
      double* tr = trace + (size_t)t * VLA_ORACLE_TRACE_WIDTH;
      tr[0] = frob(S, (size_t)dv * dk);
      tr[1] = frob(A, (size_t)dk * dk);
      tr[2] = delta;
      tr[3] = sqrt(dot(e, e, dv));
      tr[4] = dot(kh, a, dk);
      tr[5] = sqrt(dot(kh, kh, dk));
      tr[6] = sqrt(dot(a, a, dk));
      tr[7] = delta_raw;
    }
  }

  if (S_T) memcpy(S_T, S, sizeof(double) * (size_t)dv * dk);
  if (A_T) memcpy(A_T, A, sizeof(double) * (size_t)dk * dk);
  if (zkey_T) memcpy(zkey_T, zkey, sizeof(double) * dk);
  free(S); free(A); free(kh); free(u); free(z); free(a); free(e); free(kf); free(qf); free(zkey);
}

/* Returns 0 on success, 1 on an invalid argument. S0/A0/S_T/A_T/trace/opts may be NULL. */
int vla_oracle_forward_f64(const double* q, const double* k, const double* v,
                           const double* S0, const double* A0,
                           double* o, double* S_T, double* A_T, double* trace,
                           int B, int H, int T, int d_k, int d_v,
                           const vla_oracle_opts* opts) {
  if (B <= 0 || H <= 0 || T < 0 || d_k <= 0 || d_v <= 0) return 1;
  if (T > 0 && (!q || !k || !v || !o)) return 1;
  double lambda0 = opts ? opts->lambda0 : 0.1;
  double eps = opts ? opts->eps : 1e-4;
  const double* u = opts ? opts->u : NULL;
  double u_scale = opts ? opts->u_scale : 1.0;
  int refresh_period = opts ? opts->refresh_period : 0;
  double refresh_eta = opts ? opts->refresh_eta : 1e-3;
  int step_offset = opts ? opts->step_offset : 0;
  int normalise_output = opts ? opts->normalise_output : 0;
  int feature_map = opts ? opts->feature_map : 0;
  const double* zkey0 = opts ? opts->zkey0 : NULL;
  double* zkey_T = opts ? opts->zkey_T : NULL;
  if (!(lambda0 > 0.0) || !(eps > 0.0)) return 1;

  long nh = (long)B * H;
  size_t sk = (size_t)T * d_k, sv = (size_t)T * d_v;
  size_t sS = (size_t)d_v * d_k, sA = (size_t)d_k * d_k;
#pragma omp parallel for schedule(dynamic, 1)
  for (long n = 0; n < nh; ++n) {
    one_head(q + n * sk, k + n * sk, v + n * sv, u ? u + n * sk : NULL,
             S0 ? S0 + n * sS : NULL, A0 ? A0 + n * sA : NULL,
             o + n * sv, S_T ? S_T + n * sS : NULL, A_T ? A_T + n * sA : NULL,
             trace ? trace + (size_t)n * T * VLA_ORACLE_TRACE_WIDTH : NULL,
             T, d_k, d_v, lambda0, eps, u_scale, refresh_period, refresh_eta, step_offset, normalise_output,
             feature_map, zkey0 ? zkey0 + n * d_k : NULL, zkey_T ? zkey_T + n * d_k : NULL);
  }
  return 0;
}

/*
 * Plain (un-normalised) linear attention, the additive baseline the paper
 * contrasts VLA's state norm with (Section 2.2, eq. (linear-attn) numerator;
 * Section 4.1 "Contrast with standard linear attention"):
 *     S_t = S_{t-1} + v_t k_t^T ,  o_t = S_t q_t .
 * In the d_v x d_k orientation used here.  normS[(b*H+h)*T + t] = ||S_t||_F
 * (nullable), o nullable.  Oracle-side only: the GPU library has no such path.
 */
int vla_oracle_linear_attention_f64(const double* q, const double* k, const double* v,
                                    double* o, double* S_T, double* normS,
                                    int B, int H, int T, int d_k, int d_v) {
  if (B <= 0 || H <= 0 || T < 0 || d_k <= 0 || d_v <= 0) return 1;
  long nh = (long)B * H;
#pragma omp parallel for schedule(dynamic, 1)
  for (long n = 0; n < nh; ++n) {
    double* S = (double*)calloc((size_t)d_v * d_k, sizeof(double));
    for (int t = 0; t < T; ++t) {
      const double* kt = k + ((size_t)n * T + t) * d_k;
      const double* vt = v + ((size_t)n * T + t) * d_v;
      for (int i = 0; i < d_v; ++i)
        for (int j = 0; j < d_k; ++j) S[(size_t)i * d_k + j] += vt[i] * kt[j];
      if (o && q) matvec(S, q + ((size_t)n * T + t) * d_k, o + ((size_t)n * T + t) * d_v, d_v, d_k);
      if (normS) normS[(size_t)n * T + t] = frob(S, (size_t)d_v * d_k);
    }
    if (S_T) memcpy(S_T + (size_t)n * d_v * d_k, S, sizeof(double) * (size_t)d_v * d_k);
    free(S);
  }
  return 0;
}

int vla_oracle_trace_width(void) { return VLA_ORACLE_TRACE_WIDTH; }

int vla_oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
