/*
 * CPU fp64 oracle for the norm-test statistics pass and the AdamW update.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  Nothing in the product path may call it,
 * and it shares no code, header, table or constant with the HIP sources.
 *
 * What it computes, for J gradient vectors g_1..g_J of length d
 * (the workers' minibatch gradients of Sec. 3.2, or per-sample gradients of
 * Sec. 3.1):
 *
 *   mean gradient            gbar_i = (1/J) sum_j g_j[i]            (Sec. 3.2; Alg. 1 "batch gradient")
 *   A = sum_j ||g_j||^2,  B = ||sum_j g_j||^2,  C = sum_j ||g_j - gbar||^2
 *   ||gbar||^2 = B / J^2
 *   ||Var||_1  = C / (J - ddof)    ddof = 0: the DDP-Norm estimator of Sec. 3.2 / Alg. 1
 *                                  ddof = 1: the sample variance under Eq. (2)
 *   T = ||Var||_1 / (eta^2 ||gbar||^2)                              (Alg. 1, test statistic)
 *   decision: grow iff T > b_k, then round up through micro-batch,
 *             minibatch and global batch                            (Alg. 1, the If branch)
 *   AdamW with bias correction and decoupled weight decay           (Alg. 1, last five updates)
 *
 * Every floating-point step is fp64.  Inputs are the exact bit patterns the
 * GPU sees (fp32 or bfloat16 gradients, fp32 w/m/v) widened exactly.
 * Sums over coordinates use Neumaier compensation so that the result does
 * not depend on d to any visible degree; there is no blocking or reordering.
 *
 * Pins (tests/test_oracle_pins.py): the identity C = A - B/J, zero variance
 * for identical rows, Gaussian closed forms, exact rational brute force on
 * tiny inputs, numpy column variance, a library AdamW run over several steps,
 * the k = 1 sign-step closed form, and a hand-computed worked example under
 * tests/golden/.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

enum { NTO_F32 = 0, NTO_BF16 = 1 };

/* status bits reported by nto_decide */
enum {
  NTO_NONFINITE = 1u,      /* a sum is NaN or Inf: do not grow on garbage          */
  NTO_ZERO_GRAD_NORM = 2u, /* ||gbar||^2 == 0: T is 0/0 or +inf                    */
  NTO_CLAMPED = 4u,        /* the rounded batch size was cut to the maximum        */
  NTO_T_SATURATED = 16u    /* T too large for an integer batch size: treated as inf */
};

typedef struct {
  double gbar_sq;  /* ||gbar||^2                 */
  double var_l1;   /* ||Var||_1 = C/(J - ddof)   */
  double T;        /* test statistic             */
  int64_t next_b;  /* b_{k+1}                    */
  int32_t pass;    /* 1 iff not (T > b_k)        */
  uint32_t status;
} nto_decision;

static double widen(const void *base, int dtype, int64_t idx) {
  if (dtype == NTO_F32) {
    float f;
    memcpy(&f, (const char *)base + 4 * idx, 4);
    return (double)f;
  } else {
    /* bfloat16 is the upper half of an IEEE binary32 */
    uint16_t h;
    uint32_t u;
    float f;
    memcpy(&h, (const char *)base + 2 * idx, 2);
    u = (uint32_t)h << 16;
    memcpy(&f, &u, 4);
    return (double)f;
  }
}

/* running compensated sum: value is s[0] + s[1] */
static void csum_add(double *s, double x) {
  double t = s[0] + x;
  if (fabs(s[0]) >= fabs(x))
    s[1] += (s[0] - t) + x;
  else
    s[1] += (x - t) + s[0];
  s[0] = t;
}

/*
 * Accumulate A, B, C over n coordinates into acc[6] =
 * {A, A_comp, B, B_comp, C, C_comp}.  Row j of the gradient matrix starts at
 * element j*ld of `grads`.  The caller zeroes acc before the first call and may
 * call again with the next range of coordinates; the value of a sum is
 * acc[2k] + acc[2k+1].
 */
int nto_stats(const void *grads, int dtype, int64_t J, int64_t ld, int64_t n, double *acc) {
  if (!grads || !acc || J < 1 || n < 0 || ld < n || (dtype != NTO_F32 && dtype != NTO_BF16)) return -1;
  for (int64_t i = 0; i < n; ++i) {
    double s = 0.0, a = 0.0, c = 0.0, gbar;
    for (int64_t j = 0; j < J; ++j) {
      double g = widen(grads, dtype, j * ld + i);
      s += g;
      a += g * g;
    }
    gbar = s / (double)J;
    for (int64_t j = 0; j < J; ++j) {
      double r = widen(grads, dtype, j * ld + i) - gbar;
      c += r * r;
    }
    csum_add(acc + 0, a);
    csum_add(acc + 2, s * s);
    csum_add(acc + 4, c);
  }
  return 0;
}

/*
 * From the three sums to the test statistic and the next batch size.
 * round_to is J*M, the product of the number of workers and of accumulation
 * steps: ceil(ceil(T)/(J*M)) * M * J is the composition of Alg. 1's three
 * rounding lines.  round_to = 1 gives the plain ceiling rule of Sec. 3.1.
 * b_max > 0 caps the result (Sec. 5, maximum global batch size) but never
 * below b_k, since Alg. 1 never shrinks the batch.
 */
int nto_decide(double A, double B, double C, int64_t J, double eta, int64_t b_k, int64_t b_max,
               int64_t round_to, int32_t ddof, nto_decision *out) {
  double Jd = (double)J, T;
  int64_t cap;
  if (!out || J < 1 || J - ddof < 1 || !(eta > 0.0) || b_k < 1 || b_max < 0 || round_to < 1 ||
      round_to > ((int64_t)1 << 31) || (ddof != 0 && ddof != 1))
    return -1; /* the bound on round_to keeps q * round_to below 2^63 for every t < 2^62 */
  cap = (b_max > 0 && b_max > b_k) ? b_max : b_k; /* value taken when T is infinite */
  out->status = 0;
  out->gbar_sq = B / (Jd * Jd);
  out->var_l1 = C / (double)(J - ddof);
  out->pass = 1;
  out->next_b = b_k;
  if (!isfinite(A) || !isfinite(B) || !isfinite(C)) {
    out->status |= NTO_NONFINITE;
    out->T = NAN;
    return 0;
  }
  if (out->gbar_sq == 0.0) {
    out->status |= NTO_ZERO_GRAD_NORM;
    if (C == 0.0) {
      out->T = NAN; /* 0/0: nothing to test */
    } else {
      out->T = INFINITY;
      out->pass = 0;
      out->next_b = cap;
    }
    return 0;
  }
  T = out->var_l1 / (eta * eta * out->gbar_sq);
  out->T = T;
  if (T > (double)b_k) {
    out->pass = 0;
    if (!(T < 4611686018427387904.0)) { /* 2^62 */
      out->status |= NTO_T_SATURATED;
      out->next_b = cap;
    } else {
      int64_t t = (int64_t)ceil(T);
      int64_t q = t / round_to + (t % round_to != 0);
      int64_t nb = q * round_to;
      if (b_max > 0 && nb > b_max) {
        nb = b_max;
        out->status |= NTO_CLAMPED;
      }
      if (nb < b_k) nb = b_k;
      out->next_b = nb;
    }
  }
  return 0;
}

/*
 * Splitting a global batch size over J workers, M accumulation steps and a micro-batch size that has a
 * maximum (hyper-parameter tables: base micro-batch 4, maximum micro-batch 8, base accumulation steps 16,
 * data-parallel size 4, base global batch 256, maximum 8192).  Alg. 1 keeps M fixed and lets the
 * micro-batch grow; the paper does not say what happens at the maximum micro-batch size.  Reading taken:
 * keep the base M while the micro-batch fits, otherwise take the fewest accumulation steps for which it
 * fits, then the smallest micro-batch that covers b:
 *   M = max(M_base, ceil(b / (J * micro_max))),  micro = ceil(b / (J * M)),  global = J * M * micro >= b.
 */
int nto_resplit(int64_t b, int64_t J, int64_t M_base, int64_t micro_max, int64_t *micro, int64_t *M,
                int64_t *global) {
  int64_t per_worker, m, mb;
  if (b < 1 || J < 1 || M_base < 1 || micro_max < 1 || !micro || !M || !global) return -1;
  per_worker = b / J + (b % J != 0);
  m = per_worker / micro_max + (per_worker % micro_max != 0);
  if (m < M_base) m = M_base;
  mb = b / (J * m) + (b % (J * m) != 0);
  *micro = mb;
  *M = m;
  *global = J * m * mb;
  return 0;
}

/*
 * Which steps run the test (Sec. 5, training specifications; "Test interval" in the hyper-parameter tables).
 * Two rules are stated: the test is performed at a fixed interval of steps rather than at every step, and it
 * is no longer performed once the global batch size has reached its maximum.  Reading taken where the text is
 * silent: steps are counted from 1 and the first step tests, so step k tests when (k - 1) is a multiple of the
 * interval; "reached" means b_k >= b_max (a test could not enlarge the batch any more), b_max = 0 meaning no
 * maximum.  Returns 1 if step k runs the test, 0 if not, -1 for invalid arguments.
 */
int nto_test_due(int64_t step, int64_t interval, int64_t b_k, int64_t b_max) {
  if (step < 1 || interval < 1 || b_k < 1 || b_max < 0) return -1;
  if (b_max > 0 && b_k >= b_max) return 0;
  return (step - 1) % interval == 0 ? 1 : 0;
}

/*
 * Coordinate-wise form of the test.  The analysis (Sec. 4, Prop. 1; App. B remark) asks the norm-test
 * condition of every coordinate i separately; with the same estimators as the aggregate test this reads
 *   Var_i / b_k <= eta^2 gbar_i^2,   Var_i = sum_j (g_j[i] - gbar_i)^2 / (J - ddof),
 * and a coordinate fails when the inequality is violated strictly (as T > b_k in Alg. 1).  The paper
 * does not run this variant (Sec. 5) and prints no batch-size rule for it, so only the count of failing
 * coordinates is defined here.  out[0] += coordinates that fail by more than the relative band,
 * out[1] += coordinates within the band of equality (either answer is acceptable for an fp32 kernel),
 * out[2] += coordinates that pass by more than the band.  band = 0 gives the plain fp64 decision
 * (equality counts as pass).
 */
int nto_coord_test(const void *grads, int dtype, int64_t J, int64_t ld, int64_t n, double eta, int64_t b_k,
                   int32_t ddof, double band, int64_t *out) {
  if (!grads || !out || J < 1 || J - ddof < 1 || n < 0 || ld < n || !(eta > 0.0) || b_k < 1 || band < 0.0 ||
      (dtype != NTO_F32 && dtype != NTO_BF16) || (ddof != 0 && ddof != 1))
    return -1;
  for (int64_t i = 0; i < n; ++i) {
    double s = 0.0, c = 0.0, gbar, var, rhs;
    for (int64_t j = 0; j < J; ++j) s += widen(grads, dtype, j * ld + i);
    gbar = s / (double)J;
    for (int64_t j = 0; j < J; ++j) {
      double r = widen(grads, dtype, j * ld + i) - gbar;
      c += r * r;
    }
    var = c / (double)(J - ddof);
    rhs = eta * eta * (double)b_k * gbar * gbar;
    if (var > rhs * (1.0 + band))
      out[0] += 1;
    else if (band > 0.0 && rhs > 0.0 && var >= rhs * (1.0 - band))
      out[1] += 1;
    else
      out[2] += 1;
  }
  return 0;
}

/*
 * Largest violation of the coordinate-wise condition (Sec. 4, Prop. 1, with the estimators of the aggregate
 * test): the maximum over coordinates i of
 *   rho_i = Var_i / (eta^2 b_k gbar_i^2),   Var_i = sum_j (g_j[i] - gbar_i)^2 / (J - ddof),
 * so that coordinate i fails exactly when rho_i > 1, and max_i rho_i <= 1 means every coordinate passes.
 * Conventions where the quotient is not defined: a coordinate with no spread (Var_i = 0) has rho_i = 0
 * whatever its mean (0 > 0 is false: it passes); a coordinate with spread and a zero mean has rho_i = +inf.
 * *out is a running maximum: the caller sets it to 0 before the first range of coordinates and may call again
 * with further ranges (the maximum over shards is the maximum of the shards' values).
 */
int nto_coord_max_ratio(const void *grads, int dtype, int64_t J, int64_t ld, int64_t n, double eta, int64_t b_k,
                        int32_t ddof, double *out) {
  if (!grads || !out || J < 1 || J - ddof < 1 || n < 0 || ld < n || !(eta > 0.0) || b_k < 1 ||
      (dtype != NTO_F32 && dtype != NTO_BF16) || (ddof != 0 && ddof != 1))
    return -1;
  for (int64_t i = 0; i < n; ++i) {
    double total = 0.0, spread = 0.0, mean, variance, rho;
    for (int64_t j = 0; j < J; ++j) total += widen(grads, dtype, j * ld + i);
    mean = total / (double)J;
    for (int64_t j = 0; j < J; ++j) {
      double dev = widen(grads, dtype, j * ld + i) - mean;
      spread += dev * dev;
    }
    variance = spread / (double)(J - ddof);
    if (variance == 0.0)
      rho = 0.0;
    else if (mean == 0.0)
      rho = INFINITY;
    else
      rho = variance / (eta * eta * (double)b_k * mean * mean);
    if (rho > *out) *out = rho;
  }
  return 0;
}

/*
 * Global-norm gradient clipping, used in the paper's runs (Sec. 5, training specifications; the
 * hyper-parameter tables list "gradient clipping 1.0") but not part of Alg. 1.  The paper gives no
 * formula; this is the usual convention: the whole gradient is scaled by
 *   min(1, max_norm / (||gbar|| + 1e-6)).
 * max_norm <= 0 means no clipping.
 */
double nto_clip_coef(double gbar_sq, double max_norm) {
  double c;
  if (!(max_norm > 0.0)) return 1.0;
  c = max_norm / (sqrt(gbar_sq) + 1e-6);
  return c < 1.0 ? c : 1.0;
}

/*
 * AdamW on the mean gradient for n coordinates (Alg. 1):
 *   m' = beta1 m + (1-beta1) gbar          v' = beta2 v + (1-beta2) gbar^2
 *   mhat = m'/(1-beta1^k)                  vhat = v'/(1-beta2^k)
 *   w' = (1 - lr*wd) w - lr * mhat / (sqrt(vhat) + eps)
 * w, m, v are the fp32 state before the step; outputs stay in fp64.
 * grad_scale multiplies the mean gradient before it enters the moments (1 = Alg. 1 as written;
 * nto_clip_coef(...) = the clipped variant).  gbar_out (may be NULL) receives the unscaled mean.
 */
int nto_adamw(const void *grads, int dtype, int64_t J, int64_t ld, int64_t n, const float *w,
              const float *m, const float *v, double lr, double beta1, double beta2, double eps,
              double wd, int64_t step, double grad_scale, double *w_out, double *m_out, double *v_out,
              double *gbar_out) {
  double bc1, bc2;
  if (!grads || !w || !m || !v || !w_out || !m_out || !v_out || J < 1 || n < 0 || ld < n || step < 1 ||
      (dtype != NTO_F32 && dtype != NTO_BF16))
    return -1;
  bc1 = 1.0 - pow(beta1, (double)step);
  bc2 = 1.0 - pow(beta2, (double)step);
  for (int64_t i = 0; i < n; ++i) {
    double s = 0.0, gbar, g, mn, vn, mhat, vhat;
    for (int64_t j = 0; j < J; ++j) s += widen(grads, dtype, j * ld + i);
    gbar = s / (double)J;
    g = grad_scale * gbar;
    mn = beta1 * (double)m[i] + (1.0 - beta1) * g;
    vn = beta2 * (double)v[i] + (1.0 - beta2) * g * g;
    mhat = mn / bc1;
    vhat = vn / bc2;
    w_out[i] = (1.0 - lr * wd) * (double)w[i] - lr * mhat / (sqrt(vhat) + eps);
    m_out[i] = mn;
    v_out[i] = vn;
    if (gbar_out) gbar_out[i] = gbar;
  }
  return 0;
}
