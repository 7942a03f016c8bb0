/*
 * npd_oracle.c -- float64 CPU oracle for the packed knowledge-distillation loss of
 * Near-Policy Distillation (NPD).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a slow, plain statement of what the GPU
 * library must compute and shares no code with it.  Only the tests, the smoke
 * check and the benchmark's CPU-baseline leg may call it; the product path never
 * does.
 *
 * Everything here is the textbook definition written out in double precision:
 *   - student distribution   p_S = Softmax(O_S / tau)           (Alg. 1, "Compute Probs")
 *   - teacher distribution   p_T = Softmax(O_T / tau)           (Alg. 1, "Compute Probs";
 *                            with a top-k record the softmax runs over the k stored
 *                            entries only, Sec. 3.1 "Teacher Logits via Packed
 *                            Parallel Prefill")
 *   - KD loss per position   sum_{c in support} p_T(c) log(p_T(c)/p_S(c))   (Eq. 2)
 *   - CE loss per position   -log Softmax(O)[label]             (L_CE of Eq. 1; the
 *                            sequence loss L_theta of Eq. 3)
 *   - gradient of Eq. 2 with respect to the student logits (implied by the
 *     parameter update of Alg. 1): (1/tau) * (p_S(c) - p_T(c) [c in support])
 *     (p_T sums to 1 over its support, by construction of the softmax)
 *   - gradient of the composite loss of Eq. 1, L_total = (1 - lambda) L_CE + lambda L_KD:
 *     the KD gradient times grad_scale plus ce_grad_scale * (Softmax(O_S)(c) - [c == label])
 *     (the caller sets grad_scale = lambda * w and ce_grad_scale = (1 - lambda) * w)
 *   - the other token-level divergences that the Related Works section names next to the forward KL
 *     of Eq. 2 (the paper defines none of them; the definitions are those of the works it cites):
 *     reverse KL  KL(p_S || p_T), skew KL  KL(p_T || alpha p_T + (1 - alpha) p_S) and skew reverse KL
 *     KL(p_S || (1 - alpha) p_T + alpha p_S), each with its gradient with respect to the student logits
 *   - per-sample reduction over cu_seqlens under the response mask
 *   - IFD (Eq. 3), Delta-IFD (Eq. 4) and the three curation zones of Sec. 3.2
 *   - the policy-latency monitor of the appendix ("Analysis of Policy Latency": mean
 *     D_KL(pi_learner || pi_generator) of a step against the near-policy bound epsilon) and
 *     the perplexity of a sample (the PPL filter of the data-filter ablation)
 *
 * The temperature tau divides student and teacher logits alike; tau = 1 is Eq. 2
 * exactly.  No tau^2 factor is applied (a caller folds it into grad_scale).
 *
 * No blocking, no fusion, no online tricks: two-pass log-sum-exp (maximum first,
 * then the sum), sums in index order.
 *
 * Parity pins: every function below is pinned by tests/test_oracle_pins.py against
 * closed forms, library routines in float64, finite differences and brute force.
 * What no pin can reach is convention rather than arithmetic (no tau^2, top-k
 * renormalisation, mean rather than sum in Eq. 3): the paper prints no worked
 * example, so those readings are "parity unpinned" beyond self-consistency.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* zone codes of Sec. 3.2 */
enum { ZONE_DEGENERATE = 0, ZONE_PROXIMAL = 1, ZONE_DISCONNECT = 2, ZONE_INVALID = 3 };

int npd_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* bf16 is the upper half of an IEEE binary32: the conversion to double is exact. */
static double bf16_to_double(uint16_t h) {
  uint32_t u = ((uint32_t)h) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

/* log sum_i exp(a_i), two passes. */
static double logsumexp(const double *a, int64_t n) {
  double mx = -INFINITY;
  for (int64_t i = 0; i < n; ++i)
    if (a[i] > mx) mx = a[i];
  if (isinf(mx) && mx < 0) return -INFINITY; /* all -inf: empty distribution */
  double z = 0.0;
  for (int64_t i = 0; i < n; ++i) z += exp(a[i] - mx);
  return mx + log(z);
}

/* CE loss of one position: logsumexp(o) - o[label]  (natural log, no temperature). */
static double row_nll(const double *o, int64_t V, int32_t label) {
  if (label < 0 || label >= V) return NAN;
  return logsumexp(o, V) - o[label];
}

/*
 * Adds the gradient of the CE loss of one position (L_CE of Eq. 1, no temperature) to grad:
 * ce_scale * (Softmax(s)(c) - [c == label]).  An out-of-range label poisons the row with NaN.
 */
static void row_add_ce_grad(const double *s, int64_t V, int32_t label, double ce_scale, double *grad) {
  if (label < 0 || label >= V) {
    for (int64_t c = 0; c < V; ++c) grad[c] = NAN;
    return;
  }
  const double lse = logsumexp(s, V);
  for (int64_t c = 0; c < V; ++c) grad[c] += ce_scale * (exp(s[c] - lse) - (c == label ? 1.0 : 0.0));
}

/*
 * One position, dense teacher.  s, t: V logits each.  Outputs (any may be NULL):
 * kd = Eq. 2 over the full vocabulary, grad[V] = grad_scale * d kd / d s.
 * a, b are caller-provided work rows of V doubles.
 */
static void row_kd_dense(const double *s, const double *t, int64_t V, double tau, double grad_scale,
                         double *a, double *b, double *kd, double *grad) {
  for (int64_t c = 0; c < V; ++c) a[c] = s[c] / tau;
  for (int64_t c = 0; c < V; ++c) b[c] = t[c] / tau;
  const double lse_a = logsumexp(a, V);
  const double lse_b = logsumexp(b, V);
  double acc = 0.0;
  for (int64_t c = 0; c < V; ++c) {
    const double logp_t = b[c] - lse_b;
    const double logp_s = a[c] - lse_a;
    const double p_t = exp(logp_t);
    if (p_t > 0.0) acc += p_t * (logp_t - logp_s);
  }
  if (kd) *kd = acc;
  if (grad) {
    for (int64_t c = 0; c < V; ++c) {
      const double p_s = exp(a[c] - lse_a);
      const double p_t = exp(b[c] - lse_b);
      grad[c] = grad_scale * (1.0 / tau) * (p_s - p_t);
    }
  }
}

/* divergences between the teacher and student distributions of one position */
enum { DIV_FORWARD_KL = 0, DIV_REVERSE_KL = 1, DIV_SKEW_KL = 2, DIV_SKEW_REVERSE_KL = 3 };

/*
 * One position, dense teacher, any of the divergences above (Related Works: reverse KL, skew KL).
 * With p_S = Softmax(s / tau), p_T = Softmax(t / tau):
 *   forward       D = sum_c p_T log(p_T / p_S)                                   (Eq. 2)
 *   reverse       D = sum_c p_S log(p_S / p_T)
 *   skew          D = sum_c p_T log(p_T / m),  m = alpha p_T + (1 - alpha) p_S
 *   skew reverse  D = sum_c p_S log(p_S / m),  m = (1 - alpha) p_T + alpha p_S
 * The gradient follows from the chain rule through the softmax: with u_c = dD / d p_S(c),
 *   dD / d s_j = (1 / tau) p_S(j) (u_j - sum_c p_S(c) u_c),
 *   forward: u = -p_T / p_S;  reverse: u = log(p_S / p_T) + 1;
 *   skew: u = -(1 - alpha) p_T / m;  skew reverse: u = log(p_S / m) + 1 - alpha p_S / m.
 * a, b, u are caller-provided work rows of V doubles.
 */
static void row_div_dense(const double *s, const double *t, int64_t V, double tau, double grad_scale, int divergence,
                          double alpha, double *a, double *b, double *u, double *kd, double *grad) {
  if (divergence == DIV_FORWARD_KL) {
    row_kd_dense(s, t, V, tau, grad_scale, a, b, kd, grad);
    return;
  }
  for (int64_t c = 0; c < V; ++c) a[c] = s[c] / tau;
  for (int64_t c = 0; c < V; ++c) b[c] = t[c] / tau;
  const double lse_a = logsumexp(a, V);
  const double lse_b = logsumexp(b, V);
  double acc = 0.0;
  for (int64_t c = 0; c < V; ++c) {
    const double logp_s = a[c] - lse_a, logp_t = b[c] - lse_b;
    const double p_s = exp(logp_s), p_t = exp(logp_t);
    if (divergence == DIV_REVERSE_KL) {
      if (p_s > 0.0) acc += p_s * (logp_s - logp_t);
      u[c] = p_s > 0.0 ? logp_s - logp_t + 1.0 : 0.0; /* p_S = 0: no term, and p_S (u - ubar) = 0 whatever u is */
    } else if (divergence == DIV_SKEW_KL) {
      const double m = alpha * p_t + (1.0 - alpha) * p_s;
      if (p_t > 0.0) acc += p_t * (logp_t - log(m));
      u[c] = m > 0.0 ? -(1.0 - alpha) * p_t / m : 0.0;
    } else {
      const double m = (1.0 - alpha) * p_t + alpha * p_s;
      if (p_s > 0.0) acc += p_s * (logp_s - log(m));
      u[c] = p_s > 0.0 ? logp_s - log(m) + 1.0 - alpha * p_s / m : 0.0;
    }
  }
  if (kd) *kd = acc;
  if (grad) {
    double ubar = 0.0;
    for (int64_t c = 0; c < V; ++c) ubar += exp(a[c] - lse_a) * u[c];
    for (int64_t c = 0; c < V; ++c) grad[c] = grad_scale * (1.0 / tau) * exp(a[c] - lse_a) * (u[c] - ubar);
  }
}

/*
 * One position, top-k teacher record: idx[k] vocabulary ids (unique), val[k] the
 * stored teacher values (logits or log-probabilities: the softmax below is shift
 * invariant).  p_T is the softmax of val/tau over the k entries; p_S is the
 * full-vocabulary softmax of s/tau.  Returns 0, or 1 if an index is out of range
 * (outputs are then NaN).
 */
static int row_kd_topk(const double *s, int64_t V, const int32_t *idx, const double *val, int32_t k,
                       double tau, double grad_scale, double *a, double *b, double *kd, double *grad) {
  for (int32_t j = 0; j < k; ++j) {
    if (idx[j] < 0 || idx[j] >= V) {
      if (kd) *kd = NAN;
      if (grad)
        for (int64_t c = 0; c < V; ++c) grad[c] = NAN;
      return 1;
    }
  }
  for (int64_t c = 0; c < V; ++c) a[c] = s[c] / tau;
  for (int32_t j = 0; j < k; ++j) b[j] = val[j] / tau;
  const double lse_a = logsumexp(a, V);
  const double lse_b = logsumexp(b, k);
  double acc = 0.0;
  for (int32_t j = 0; j < k; ++j) {
    const double logp_t = b[j] - lse_b;
    const double logp_s = a[idx[j]] - lse_a;
    const double p_t = exp(logp_t);
    if (p_t > 0.0) acc += p_t * (logp_t - logp_s);
  }
  if (kd) *kd = acc;
  if (grad) {
    for (int64_t c = 0; c < V; ++c) grad[c] = grad_scale * (1.0 / tau) * exp(a[c] - lse_a);
    for (int32_t j = 0; j < k; ++j)
      grad[idx[j]] -= grad_scale * (1.0 / tau) * exp(b[j] - lse_b);
  }
  return 0;
}

/* ------------------------------------------------------------------------- */
/* Entry points on double logits (used by the pin tests).                     */
/* ------------------------------------------------------------------------- */

/*
 * Dense-teacher KD over T positions.  s, t: [T, V] doubles, row-major, contiguous.
 * labels may be NULL (then nll_s / nll_t must be NULL and ce_grad_scale 0); mask is required.
 * Masked positions give kd = nll = 0 and a zero gradient row.
 * Outputs (each may be NULL): kd[T], nll_s[T], nll_t[T], lse_s[T] (log-sum-exp of the
 * raw student logits, tau = 1), grad[T, V].
 */
void npd_oracle_kd_dense_f64(int64_t T, int64_t V, const double *s, const double *t, const int32_t *labels,
                             const uint8_t *mask, double tau, double grad_scale, double ce_grad_scale, double *kd,
                             double *nll_s, double *nll_t, double *lse_s, double *grad) {
#pragma omp parallel
  {
    double *a = (double *)malloc(sizeof(double) * (size_t)V);
    double *b = (double *)malloc(sizeof(double) * (size_t)V);
#pragma omp for schedule(dynamic, 1)
    for (int64_t r = 0; r < T; ++r) {
      double *g = grad ? grad + r * V : NULL;
      if (!mask[r]) {
        if (kd) kd[r] = 0.0;
        if (nll_s) nll_s[r] = 0.0;
        if (nll_t) nll_t[r] = 0.0;
        if (lse_s) lse_s[r] = 0.0;
        if (g)
          for (int64_t c = 0; c < V; ++c) g[c] = 0.0;
        continue;
      }
      const double *sr = s + r * V, *tr = t + r * V;
      row_kd_dense(sr, tr, V, tau, grad_scale, a, b, kd ? kd + r : NULL, g);
      if (g && ce_grad_scale != 0.0) row_add_ce_grad(sr, V, labels[r], ce_grad_scale, g);
      if (nll_s) nll_s[r] = row_nll(sr, V, labels[r]);
      if (nll_t) nll_t[r] = row_nll(tr, V, labels[r]);
      if (lse_s) lse_s[r] = logsumexp(sr, V);
    }
    free(a);
    free(b);
  }
}

/*
 * Top-k-teacher KD over T positions.  s: [T, V]; idx: [T, k]; val: [T, k].
 * Returns the number of unmasked positions that held an out-of-range index.
 */
int64_t npd_oracle_kd_topk_f64(int64_t T, int64_t V, int32_t k, const double *s, const int32_t *idx,
                               const double *val, const int32_t *labels, const uint8_t *mask, double tau,
                               double grad_scale, double ce_grad_scale, double *kd, double *nll_s, double *lse_s,
                               double *grad) {
  int64_t bad = 0;
#pragma omp parallel reduction(+ : bad)
  {
    double *a = (double *)malloc(sizeof(double) * (size_t)V);
    double *b = (double *)malloc(sizeof(double) * (size_t)(k > 0 ? k : 1));
#pragma omp for schedule(dynamic, 1)
    for (int64_t r = 0; r < T; ++r) {
      double *g = grad ? grad + r * V : NULL;
      if (!mask[r]) {
        if (kd) kd[r] = 0.0;
        if (nll_s) nll_s[r] = 0.0;
        if (lse_s) lse_s[r] = 0.0;
        if (g)
          for (int64_t c = 0; c < V; ++c) g[c] = 0.0;
        continue;
      }
      const double *sr = s + r * V;
      bad += row_kd_topk(sr, V, idx + r * (int64_t)k, val + r * (int64_t)k, k, tau, grad_scale, a, b,
                         kd ? kd + r : NULL, g);
      if (g && ce_grad_scale != 0.0) row_add_ce_grad(sr, V, labels[r], ce_grad_scale, g);
      if (nll_s) nll_s[r] = row_nll(sr, V, labels[r]);
      if (lse_s) lse_s[r] = logsumexp(sr, V);
    }
    free(a);
    free(b);
  }
  return bad;
}

/* Forward-only CE loss per position of any logits o[T, V] (tau = 1). */
void npd_oracle_nll_f64(int64_t T, int64_t V, const double *o, const int32_t *labels, const uint8_t *mask,
                        double *nll, double *lse) {
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t r = 0; r < T; ++r) {
    if (!mask[r]) {
      if (nll) nll[r] = 0.0;
      if (lse) lse[r] = 0.0;
      continue;
    }
    if (nll) nll[r] = row_nll(o + r * V, V, labels[r]);
    if (lse) lse[r] = logsumexp(o + r * V, V);
  }
}

/* ------------------------------------------------------------------------- */
/* Entry points on bf16 logits (what the GPU library is compared against).   */
/* Each row is converted exactly to double and handed to the same row code.  */
/* Strides are in elements.  grad is [T, V] doubles, contiguous.             */
/* ------------------------------------------------------------------------- */

void npd_oracle_kd_dense_bf16(int64_t T, int64_t V, const uint16_t *s, int64_t s_stride, const uint16_t *t,
                              int64_t t_stride, const int32_t *labels, const uint8_t *mask, double tau,
                              double grad_scale, double ce_grad_scale, double *kd, double *nll_s, double *nll_t,
                              double *lse_s, double *grad) {
#pragma omp parallel
  {
    double *sr = (double *)malloc(sizeof(double) * (size_t)V);
    double *tr = (double *)malloc(sizeof(double) * (size_t)V);
    double *a = (double *)malloc(sizeof(double) * (size_t)V);
    double *b = (double *)malloc(sizeof(double) * (size_t)V);
#pragma omp for schedule(dynamic, 1)
    for (int64_t r = 0; r < T; ++r) {
      double *g = grad ? grad + r * V : NULL;
      if (!mask[r]) {
        if (kd) kd[r] = 0.0;
        if (nll_s) nll_s[r] = 0.0;
        if (nll_t) nll_t[r] = 0.0;
        if (lse_s) lse_s[r] = 0.0;
        if (g)
          for (int64_t c = 0; c < V; ++c) g[c] = 0.0;
        continue;
      }
      for (int64_t c = 0; c < V; ++c) sr[c] = bf16_to_double(s[r * s_stride + c]);
      for (int64_t c = 0; c < V; ++c) tr[c] = bf16_to_double(t[r * t_stride + c]);
      row_kd_dense(sr, tr, V, tau, grad_scale, a, b, kd ? kd + r : NULL, g);
      if (g && ce_grad_scale != 0.0) row_add_ce_grad(sr, V, labels[r], ce_grad_scale, g);
      if (nll_s) nll_s[r] = row_nll(sr, V, labels[r]);
      if (nll_t) nll_t[r] = row_nll(tr, V, labels[r]);
      if (lse_s) lse_s[r] = logsumexp(sr, V);
    }
    free(sr);
    free(tr);
    free(a);
    free(b);
  }
}

/*
 * Dense-teacher distillation with a selectable divergence (0 forward KL, 1 reverse KL, 2 skew KL, 3 skew reverse KL;
 * alpha is the skew coefficient, ignored by 0 and 1).  Same conventions as npd_oracle_kd_dense_f64; outputs kd[T] and
 * grad[T, V] (each may be NULL); labels are needed only when ce_grad_scale != 0.
 */
void npd_oracle_div_dense_f64(int64_t T, int64_t V, const double *s, const double *t, const int32_t *labels,
                              const uint8_t *mask, double tau, double grad_scale, double ce_grad_scale,
                              int32_t divergence, double alpha, double *kd, double *grad) {
#pragma omp parallel
  {
    double *a = (double *)malloc(sizeof(double) * (size_t)V);
    double *b = (double *)malloc(sizeof(double) * (size_t)V);
    double *u = (double *)malloc(sizeof(double) * (size_t)V);
#pragma omp for schedule(dynamic, 1)
    for (int64_t r = 0; r < T; ++r) {
      double *g = grad ? grad + r * V : NULL;
      if (!mask[r]) {
        if (kd) kd[r] = 0.0;
        if (g)
          for (int64_t c = 0; c < V; ++c) g[c] = 0.0;
        continue;
      }
      row_div_dense(s + r * V, t + r * V, V, tau, grad_scale, divergence, alpha, a, b, u, kd ? kd + r : NULL, g);
      if (g && ce_grad_scale != 0.0) row_add_ce_grad(s + r * V, V, labels[r], ce_grad_scale, g);
    }
    free(a);
    free(b);
    free(u);
  }
}

void npd_oracle_div_dense_bf16(int64_t T, int64_t V, const uint16_t *s, int64_t s_stride, const uint16_t *t,
                               int64_t t_stride, const int32_t *labels, const uint8_t *mask, double tau,
                               double grad_scale, double ce_grad_scale, int32_t divergence, double alpha, double *kd,
                               double *grad) {
#pragma omp parallel
  {
    double *sr = (double *)malloc(sizeof(double) * (size_t)V);
    double *tr = (double *)malloc(sizeof(double) * (size_t)V);
    double *a = (double *)malloc(sizeof(double) * (size_t)V);
    double *b = (double *)malloc(sizeof(double) * (size_t)V);
    double *u = (double *)malloc(sizeof(double) * (size_t)V);
#pragma omp for schedule(dynamic, 1)
    for (int64_t r = 0; r < T; ++r) {
      double *g = grad ? grad + r * V : NULL;
      if (!mask[r]) {
        if (kd) kd[r] = 0.0;
        if (g)
          for (int64_t c = 0; c < V; ++c) g[c] = 0.0;
        continue;
      }
      for (int64_t c = 0; c < V; ++c) sr[c] = bf16_to_double(s[r * s_stride + c]);
      for (int64_t c = 0; c < V; ++c) tr[c] = bf16_to_double(t[r * t_stride + c]);
      row_div_dense(sr, tr, V, tau, grad_scale, divergence, alpha, a, b, u, kd ? kd + r : NULL, g);
      if (g && ce_grad_scale != 0.0) row_add_ce_grad(sr, V, labels[r], ce_grad_scale, g);
    }
    free(sr);
    free(tr);
    free(a);
    free(b);
    free(u);
  }
}

int64_t npd_oracle_kd_topk_bf16(int64_t T, int64_t V, int32_t k, const uint16_t *s, int64_t s_stride,
                                const int32_t *idx, const float *val, const int32_t *labels,
                                const uint8_t *mask, double tau, double grad_scale, double ce_grad_scale, double *kd,
                                double *nll_s, double *lse_s, double *grad) {
  int64_t bad = 0;
#pragma omp parallel reduction(+ : bad)
  {
    double *sr = (double *)malloc(sizeof(double) * (size_t)V);
    double *a = (double *)malloc(sizeof(double) * (size_t)V);
    double *b = (double *)malloc(sizeof(double) * (size_t)(k > 0 ? k : 1));
    double *vr = (double *)malloc(sizeof(double) * (size_t)(k > 0 ? k : 1));
#pragma omp for schedule(dynamic, 1)
    for (int64_t r = 0; r < T; ++r) {
      double *g = grad ? grad + r * V : NULL;
      if (!mask[r]) {
        if (kd) kd[r] = 0.0;
        if (nll_s) nll_s[r] = 0.0;
        if (lse_s) lse_s[r] = 0.0;
        if (g)
          for (int64_t c = 0; c < V; ++c) g[c] = 0.0;
        continue;
      }
      for (int64_t c = 0; c < V; ++c) sr[c] = bf16_to_double(s[r * s_stride + c]);
      for (int32_t j = 0; j < k; ++j) vr[j] = (double)val[r * (int64_t)k + j];
      bad += row_kd_topk(sr, V, idx + r * (int64_t)k, vr, k, tau, grad_scale, a, b, kd ? kd + r : NULL, g);
      if (g && ce_grad_scale != 0.0) row_add_ce_grad(sr, V, labels[r], ce_grad_scale, g);
      if (nll_s) nll_s[r] = row_nll(sr, V, labels[r]);
      if (lse_s) lse_s[r] = logsumexp(sr, V);
    }
    free(sr);
    free(a);
    free(b);
    free(vr);
  }
  return bad;
}

void npd_oracle_nll_bf16(int64_t T, int64_t V, const uint16_t *o, int64_t o_stride, const int32_t *labels,
                         const uint8_t *mask, double *nll, double *lse) {
#pragma omp parallel
  {
    double *row = (double *)malloc(sizeof(double) * (size_t)V);
#pragma omp for schedule(dynamic, 1)
    for (int64_t r = 0; r < T; ++r) {
      if (!mask[r]) {
        if (nll) nll[r] = 0.0;
        if (lse) lse[r] = 0.0;
        continue;
      }
      for (int64_t c = 0; c < V; ++c) row[c] = bf16_to_double(o[r * o_stride + c]);
      if (nll) nll[r] = row_nll(row, V, labels[r]);
      if (lse) lse[r] = logsumexp(row, V);
    }
    free(row);
  }
}

/* ------------------------------------------------------------------------- */
/* Per-sample reduction over the packed layout.                               */
/* ------------------------------------------------------------------------- */

/*
 * Sample i owns the flattened positions [cu[i], cu[i+1]).  For each sample:
 * sum of x over its unmasked positions (index order), their count, and the mean
 * (0 when the count is 0).  token_to_sample (may be NULL) receives the owning
 * sample of every position, -1 for positions outside [cu[0], cu[S]).
 * Returns 0, or 1 if cu is decreasing somewhere or leaves [0, T].
 */
int npd_oracle_segment_reduce(int64_t T, int32_t S, const double *x, const uint8_t *mask, const int32_t *cu,
                              double *seg_sum, int32_t *seg_count, double *seg_mean,
                              int32_t *token_to_sample) {
  for (int32_t i = 0; i < S; ++i)
    if (cu[i] > cu[i + 1]) return 1;
  if (S > 0 && (cu[0] < 0 || cu[S] > T)) return 1;
  if (token_to_sample)
    for (int64_t p = 0; p < T; ++p) token_to_sample[p] = -1;
  for (int32_t i = 0; i < S; ++i) {
    double acc = 0.0;
    int32_t n = 0;
    for (int64_t p = cu[i]; p < cu[i + 1]; ++p) {
      if (token_to_sample) token_to_sample[p] = i;
      if (mask[p]) {
        acc += x[p];
        n += 1;
      }
    }
    if (seg_sum) seg_sum[i] = acc;
    if (seg_count) seg_count[i] = n;
    if (seg_mean) seg_mean[i] = n > 0 ? acc / (double)n : 0.0;
  }
  return 0;
}

/* ------------------------------------------------------------------------- */
/* IFD, Delta-IFD and zones.                                                  */
/* ------------------------------------------------------------------------- */

/*
 * Pair p names two packed samples: pair_cond[p] holds instruction + response (its
 * mean response loss is L(A|Q)), pair_uncond[p] holds the response alone (L(A)).
 *   IFD_M   = L_M(A|Q) / L_M(A)                  for M in {student, teacher}   (Eq. 3)
 *   Delta   = IFD_teacher - IFD_student                                         (Eq. 4)
 *   zone    = DEGENERATE if Delta < lo, DISCONNECT if Delta > hi, else PROXIMAL (Sec. 3.2;
 *             the paper's lo is 0 and hi its threshold tau); the comparison is made on
 *             Delta rounded to binary32, the precision the zone decision is specified in.
 *   INVALID when either sample has no scored position, a denominator is 0, one of the
 *             four mean losses is not finite (NaN, or an infinite loss: a response the
 *             model gives probability 0 has no difficulty ratio), or a result is not
 *             finite; IFD and Delta are then NaN.
 *   keep    = zone is PROXIMAL (and, if flag bit 0 is set, IFD_teacher <= 1, the extra
 *             condition named in the description of the proximal zone).
 * Returns the number of kept pairs.
 */
int32_t npd_oracle_delta_ifd(int32_t P, const double *mean_nll_student, const double *mean_nll_teacher,
                             const int32_t *seg_count, const int32_t *pair_cond, const int32_t *pair_uncond,
                             double lo, double hi, uint32_t flags, double *ifd_student, double *ifd_teacher,
                             double *delta, uint8_t *zone, uint8_t *keep) {
  int32_t kept = 0;
  for (int32_t p = 0; p < P; ++p) {
    const int32_t ic = pair_cond[p], iu = pair_uncond[p];
    double is = NAN, it = NAN, d = NAN;
    uint8_t z = ZONE_INVALID, kp = 0;
    const int ok_counts = seg_count[ic] > 0 && seg_count[iu] > 0;
    const int ok_means = isfinite(mean_nll_student[ic]) && isfinite(mean_nll_student[iu]) &&
                         isfinite(mean_nll_teacher[ic]) && isfinite(mean_nll_teacher[iu]);
    if (ok_counts && ok_means && mean_nll_student[iu] != 0.0 && mean_nll_teacher[iu] != 0.0) {
      is = mean_nll_student[ic] / mean_nll_student[iu];
      it = mean_nll_teacher[ic] / mean_nll_teacher[iu];
      d = it - is;
    }
    if (isfinite(is) && isfinite(it) && isfinite(d)) {
      const float d32 = (float)d;
      if (d32 < (float)lo)
        z = ZONE_DEGENERATE;
      else if (d32 > (float)hi)
        z = ZONE_DISCONNECT;
      else
        z = ZONE_PROXIMAL;
      kp = (z == ZONE_PROXIMAL);
      if ((flags & 1u) && !((float)it <= 1.0f)) kp = 0;
    } else {
      is = it = d = NAN;
    }
    if (ifd_student) ifd_student[p] = is;
    if (ifd_teacher) ifd_teacher[p] = it;
    if (delta) delta[p] = d;
    if (zone) zone[p] = z;
    if (keep) keep[p] = kp;
    kept += kp;
  }
  return kept;
}

/* ------------------------------------------------------------------------- */
/* Policy latency and perplexity.                                             */
/* ------------------------------------------------------------------------- */

/*
 * Policy latency (appendix, "Analysis of Policy Latency"): the paper tracks
 * D_KL(pi_learner || pi_generator) between the model being trained and the model that
 * generated the rollouts, and calls training near-policy while that distance stays within
 * a small threshold, D_KL <= epsilon (it reports epsilon ~ 0.10); a refresh of the rollouts
 * is due when the distance goes beyond it.
 *
 * kl_tok[p] is the KL divergence of the two next-token distributions at position p (Eq. 2's
 * form with the learner's distribution leading).  Over the packed layout:
 *   seg_mean[i], seg_count[i]  mean of kl_tok over the scored positions of sample i, their
 *                              number (mean 0 for an empty sample)
 *   batch_count                scored positions owned by any sample
 *   batch_mean                 sum of kl_tok over those positions / batch_count: the step's
 *                              D_KL, every scored token weighing the same (0 if none)
 *   return value               1 if the batch left the near-policy regime, batch_mean >
 *                              epsilon (or is not a number), else 0.  The comparison is made
 *                              on the mean rounded to binary32, the precision the decision
 *                              is specified in.
 * Returns -1 for a cu_seqlens that decreases or leaves [0, T].
 */
int npd_oracle_policy_lag(int64_t T, int32_t S, const double *kl_tok, const uint8_t *mask, const int32_t *cu,
                          double epsilon, double *seg_mean, int32_t *seg_count, double *batch_mean,
                          int64_t *batch_count) {
  for (int32_t i = 0; i < S; ++i)
    if (cu[i] > cu[i + 1]) return -1;
  if (S > 0 && (cu[0] < 0 || cu[S] > T)) return -1;
  double total = 0.0;
  int64_t n_total = 0;
  for (int32_t i = 0; i < S; ++i) {
    double acc = 0.0;
    int32_t n = 0;
    for (int64_t q = cu[i]; q < cu[i + 1]; ++q) {
      if (mask[q]) {
        acc += kl_tok[q];
        n += 1;
      }
    }
    if (seg_mean) seg_mean[i] = n > 0 ? acc / (double)n : 0.0;
    if (seg_count) seg_count[i] = n;
    total += acc;
    n_total += n;
  }
  const double mean = n_total > 0 ? total / (double)n_total : 0.0;
  if (batch_mean) *batch_mean = mean;
  if (batch_count) *batch_count = n_total;
  return !((float)mean <= (float)epsilon);
}

/*
 * Perplexity of a sample, PPL = exp(mean CE loss over its scored positions): the filter metric
 * the paper's data-filter ablation compares Delta-IFD with.  0 for an empty sample.
 */
void npd_oracle_perplexity(int32_t S, const double *mean_nll, const int32_t *seg_count, double *ppl) {
  for (int32_t i = 0; i < S; ++i) ppl[i] = seg_count[i] > 0 ? exp(mean_nll[i]) : 0.0;
}

/* ------------------------------------------------------------------------- */
/* Teacher-side top-k record (Sec. 3.1, "record only the top-k logits").      */
/* ------------------------------------------------------------------------- */

/*
 * For every scored position: the k vocabulary ids with the largest teacher logits, largest
 * first, equal logits in order of increasing id, by k plain selection scans.  val holds the
 * logits themselves, or (log_probs != 0) their log-softmax over the k selected entries, which
 * is the teacher distribution Eq. 2 uses.  Unscored positions get ids 0..k-1 and values 0.
 * t: [T, stride] bf16 bit patterns.  taken: caller-independent scratch is allocated per thread.
 */
void npd_oracle_teacher_topk_bf16(int64_t T, int64_t V, int32_t k, const uint16_t *t, int64_t t_stride,
                                  const uint8_t *mask, int log_probs, int32_t *idx, double *val) {
#pragma omp parallel
  {
    double *row = (double *)malloc(sizeof(double) * (size_t)V);
    uint8_t *taken = (uint8_t *)malloc((size_t)V);
#pragma omp for schedule(dynamic, 1)
    for (int64_t r = 0; r < T; ++r) {
      int32_t *ir = idx + r * (int64_t)k;
      double *vr = val + r * (int64_t)k;
      if (mask && !mask[r]) {
        for (int32_t j = 0; j < k; ++j) {
          ir[j] = j;
          vr[j] = 0.0;
        }
        continue;
      }
      for (int64_t c = 0; c < V; ++c) row[c] = bf16_to_double(t[r * t_stride + c]);
      memset(taken, 0, (size_t)V);
      for (int32_t j = 0; j < k; ++j) {
        int64_t best = -1;
        for (int64_t c = 0; c < V; ++c)
          if (!taken[c] && (best < 0 || row[c] > row[best])) best = c; /* first of equals wins */
        taken[best] = 1;
        ir[j] = (int32_t)best;
        vr[j] = row[best];
      }
      if (log_probs) {
        const double lse = logsumexp(vr, k);
        for (int32_t j = 0; j < k; ++j) vr[j] -= lse;
      }
    }
    free(row);
    free(taken);
  }
}
