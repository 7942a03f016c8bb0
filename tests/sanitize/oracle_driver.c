/*
 * Drives every entry point of the CPU oracle over small ragged inputs (vocabulary of 1, strides larger than
 * the row, masked rows, labels and top-k ids out of range, empty samples, k equal to the vocabulary) so that a
 * build with -fsanitize=address,undefined reports any out-of-bounds access, use of freed memory or undefined
 * arithmetic.  Values are not checked here (the pin tests do that); the exit status is 0 when nothing was reported.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int npd_oracle_threads(void);
void npd_oracle_kd_dense_f64(int64_t, int64_t, const double *, const double *, const int32_t *, const uint8_t *,
                             double, double, double, double *, double *, double *, double *, double *);
int64_t npd_oracle_kd_topk_f64(int64_t, int64_t, int32_t, const double *, const int32_t *, const double *,
                               const int32_t *, const uint8_t *, double, double, double, double *, double *,
                               double *, double *);
void npd_oracle_nll_f64(int64_t, int64_t, const double *, const int32_t *, const uint8_t *, double *, double *);
void npd_oracle_kd_dense_bf16(int64_t, int64_t, const uint16_t *, int64_t, const uint16_t *, int64_t,
                              const int32_t *, const uint8_t *, double, double, double, double *, double *,
                              double *, double *, double *);
void npd_oracle_div_dense_f64(int64_t, int64_t, const double *, const double *, const int32_t *, const uint8_t *,
                              double, double, double, int32_t, double, double *, double *);
void npd_oracle_div_dense_bf16(int64_t, int64_t, const uint16_t *, int64_t, const uint16_t *, int64_t,
                               const int32_t *, const uint8_t *, double, double, double, int32_t, double, double *,
                               double *);
int64_t npd_oracle_kd_topk_bf16(int64_t, int64_t, int32_t, const uint16_t *, int64_t, const int32_t *,
                                const float *, const int32_t *, const uint8_t *, double, double, double, double *,
                                double *, double *, double *);
void npd_oracle_nll_bf16(int64_t, int64_t, const uint16_t *, int64_t, const int32_t *, const uint8_t *, double *,
                         double *);
int npd_oracle_segment_reduce(int64_t, int32_t, const double *, const uint8_t *, const int32_t *, double *,
                              int32_t *, double *, int32_t *);
int32_t npd_oracle_delta_ifd(int32_t, const double *, const double *, const int32_t *, const int32_t *,
                             const int32_t *, double, double, uint32_t, double *, double *, double *, uint8_t *,
                             uint8_t *);
void npd_oracle_teacher_topk_bf16(int64_t, int64_t, int32_t, const uint16_t *, int64_t, const uint8_t *, int,
                                  int32_t *, double *);

static uint64_t state = 0x9e3779b97f4a7c15ull;
static double uniform(void) { /* in (-1, 1) */
  state = state * 6364136223846793005ull + 1442695040888963407ull;
  return (double)(int64_t)(state >> 11) / 4503599627370496.0 - 1.0;
}
static uint16_t to_bf16(double x) {
  float f = (float)x;
  uint32_t u;
  memcpy(&u, &f, 4);
  return (uint16_t)(u >> 16);
}
/* exact-size heap blocks: a sanitizer sees any access one element past either end */
static void *block(size_t bytes) {
  void *p = malloc(bytes ? bytes : 1);
  if (!p) exit(3);
  return p;
}

static void one_shape(int64_t T, int64_t V, int32_t k, int64_t pad) {
  const int64_t stride = V + pad;
  double *s = block(sizeof(double) * T * V), *t = block(sizeof(double) * T * V);
  uint16_t *sb = block(2 * ((T - 1) * stride + V)), *tb = block(2 * ((T - 1) * stride + V));
  int32_t *labels = block(4 * T), *idx = block(4 * T * k), *oidx = block(4 * T * k);
  double *val = block(8 * T * k), *oval = block(8 * T * k);
  float *valf = block(4 * T * k);
  uint8_t *mask = block(T);
  double *kd = block(8 * T), *nll = block(8 * T), *tnll = block(8 * T), *lse = block(8 * T);
  double *grad = block(8 * T * V);
  for (int64_t r = 0; r < T; ++r) {
    for (int64_t c = 0; c < V; ++c) {
      s[r * V + c] = 6.0 * uniform();
      t[r * V + c] = 0.8 * s[r * V + c] + 3.0 * uniform();
      sb[r * stride + c] = to_bf16(s[r * V + c]);
      tb[r * stride + c] = to_bf16(t[r * V + c]);
    }
    mask[r] = (uint8_t)(r % 3 != 1);
    labels[r] = (int32_t)((r * 7) % V);
    for (int32_t j = 0; j < k; ++j) {
      idx[r * k + j] = (int32_t)((r + j) % V); /* distinct within a row since k <= V */
      val[r * k + j] = 4.0 * uniform();
      valf[r * k + j] = (float)val[r * k + j];
    }
  }
  if (T > 2) {
    labels[0] = (int32_t)V; /* out of range at a scored position: NaN by definition, never an access */
    labels[2] = -1;
    idx[2 * k] = (int32_t)V + 5;
  }
  for (double tau = 1.0; tau < 2.5; tau += 1.0) {
    npd_oracle_kd_dense_f64(T, V, s, t, labels, mask, tau, 1.0, 0.1, kd, nll, tnll, lse, grad);
    npd_oracle_kd_dense_f64(T, V, s, t, NULL, mask, tau, 1.0, 0.0, kd, NULL, NULL, NULL, NULL);
    npd_oracle_kd_dense_bf16(T, V, sb, stride, tb, stride, labels, mask, tau, 0.5, 0.1, kd, nll, tnll, lse, grad);
    npd_oracle_kd_topk_f64(T, V, k, s, idx, val, labels, mask, tau, 1.0, 0.1, kd, nll, lse, grad);
    npd_oracle_kd_topk_bf16(T, V, k, sb, stride, idx, valf, labels, mask, tau, 1.0, 0.0, kd, nll, lse, grad);
    for (int32_t div = 0; div < 4; ++div) {
      npd_oracle_div_dense_f64(T, V, s, t, labels, mask, tau, 1.0, 0.1, div, 0.1, kd, grad);
      npd_oracle_div_dense_bf16(T, V, sb, stride, tb, stride, labels, mask, tau, 1.0, 0.0, div, 0.5, kd, NULL);
    }
  }
  npd_oracle_nll_f64(T, V, s, labels, mask, nll, lse);
  npd_oracle_nll_bf16(T, V, tb, stride, labels, mask, nll, NULL);
  npd_oracle_teacher_topk_bf16(T, V, k, tb, stride, mask, 0, oidx, oval);
  npd_oracle_teacher_topk_bf16(T, V, k, tb, stride, NULL, 1, oidx, oval);
  free(s), free(t), free(sb), free(tb), free(labels), free(idx), free(oidx), free(val), free(oval), free(valf);
  free(mask), free(kd), free(nll), free(tnll), free(lse), free(grad);
}

static void bookkeeping(void) {
  enum { T = 41, S = 7, P = 5 };
  const int32_t cu[S + 1] = {0, 0, 5, 6, 6, 30, 30, 37}; /* empty samples, a single position, an unowned tail */
  double *x = block(8 * T), *sum = block(8 * S), *mean = block(8 * S);
  uint8_t *mask = block(T);
  int32_t *cnt = block(4 * S), *owner = block(4 * T);
  for (int p = 0; p < T; ++p) x[p] = uniform(), mask[p] = (uint8_t)(p % 4 != 0);
  if (npd_oracle_segment_reduce(T, S, x, mask, cu, sum, cnt, mean, owner)) exit(4);
  if (npd_oracle_segment_reduce(T, S, x, mask, cu, NULL, NULL, NULL, NULL)) exit(4);
  if (npd_oracle_segment_reduce(T, 0, x, mask, cu, sum, cnt, mean, owner)) exit(4);
  const int32_t decreasing[3] = {0, 9, 4};
  if (!npd_oracle_segment_reduce(T, 2, x, mask, decreasing, sum, cnt, mean, owner)) exit(5);
  const int32_t beyond[2] = {0, T + 1};
  if (!npd_oracle_segment_reduce(T, 1, x, mask, beyond, sum, cnt, mean, owner)) exit(5);

  double ms[S], mt[S];
  for (int i = 0; i < S; ++i) ms[i] = 1.5 + uniform(), mt[i] = 1.5 + uniform(), cnt[i] = i % 3;
  ms[2] = 0.0, mt[4] = INFINITY;
  const int32_t pc[P] = {0, 1, 2, 4, 6}, pu[P] = {1, 2, 5, 2, 4};
  double *is = block(8 * P), *it = block(8 * P), *d = block(8 * P);
  uint8_t *zone = block(P), *keep = block(P);
  npd_oracle_delta_ifd(P, ms, mt, cnt, pc, pu, 0.0, 0.8, 0, is, it, d, zone, keep);
  npd_oracle_delta_ifd(P, ms, mt, cnt, pc, pu, -1.0, 1.0, 1, NULL, NULL, NULL, NULL, NULL);
  npd_oracle_delta_ifd(0, ms, mt, cnt, pc, pu, 0.0, 0.8, 0, is, it, d, zone, keep);
  free(x), free(sum), free(mean), free(mask), free(cnt), free(owner), free(is), free(it), free(d), free(zone);
  free(keep);
}

int main(void) {
  if (npd_oracle_threads() < 1) return 2;
  one_shape(1, 1, 1, 0);
  one_shape(5, 2, 2, 3);
  one_shape(7, 33, 33, 0);
  one_shape(9, 50, 8, 14);
  one_shape(4, 257, 64, 7);
  bookkeeping();
  puts("oracle driver finished");
  return 0;
}
