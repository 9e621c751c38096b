/*
 * CPU oracle for packed variable-length multi-head attention, fp64.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain definition the HIP
 * library is checked against.  It shares no source with the library and must
 * never be linked, imported or called by it; only tests, the smoke check and
 * the benchmark's cpu_baseline leg use it.
 *
 * What it computes, for each sequence i (rows cu[i] .. cu[i+1]-1 of the packed
 * tensors; the prefix-sum array is the paper's batch_offset, Section IV-A-1)
 * and each head h independently:
 *
 *   forward  (Eq. 1 of the paper, with the scale 1/sqrt(d_k) passed in as
 *             `scale`):   S = scale * Q K^T
 *                         P = softmax over keys of S (row-wise)
 *                         O = P V
 *                         LSE_r = log sum_j exp(S_rj)
 *   backward (the paper prints no formula; this is the derivative of Eq. 1
 *             for an upstream gradient dO):
 *                         dV = P^T dO
 *                         dP = dO V^T
 *                         D_r = sum_j P_rj dP_rj
 *                         dS = P o (dP - D)
 *                         dQ = scale * dS K
 *                         dK = scale * dS^T Q
 *
 * Only keys j < nk_i take part, where nk_i = seqused[i] if that array is
 * given (the padded baseline: every sequence occupies a fixed number of rows
 * and the keys beyond its true length are masked) and L_i otherwise.  All L_i
 * query rows are computed either way.  Rows of different sequences never
 * interact: that is what "only the valid tokens" means for attention.
 * A row with no admissible key (nk_i = 0, only possible through seqused) has
 * O = 0, LSE = -inf and contributes no gradient.
 *
 * Dropout on the attention probabilities (BERT's training configuration,
 * Section V-A; the paper does not describe it inside the attention kernel):
 * the *_dropout entry points take an explicit keep mask M (1 = kept; how it is
 * drawn is dropout_mask.py's business) and a factor c = 1 / (1 - p):
 *                         O  = (P o M c) V
 *                         dV = (P o M c)^T dO
 *                         dP = (dO V^T) o M c
 *             D, dS, dQ, dK as above (the softmax itself, and LSE, are unchanged).
 * Mask layout: sequence i, head h, query r, key j at
 * keep[keep_off[i] + (h * L_i + r) * L_i + j].
 *
 * Everything is plain loops in double precision, natural exp/log, parallel
 * over (sequence, head) only.  Build without -ffast-math.
 *
 * Tensors: [T, H, D] row-major doubles (element (t,h,c) at (t*H + h)*D + c).
 * LSE: [H, T].  Pins: tests/test_oracle_*.py (brute force, closed forms,
 * invariants, finite differences, a library softmax).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int check_cu(const int32_t *cu, int B) {
  if (!cu || B < 0 || cu[0] != 0) return 1;
  for (int i = 0; i < B; i++)
    if (cu[i + 1] < cu[i]) return 1;
  return 0;
}

/* scores of one query row against keys [0, nk) and their softmax; returns LSE */
static double softmax_row(const double *q, const double *kbase, int64_t kstride, int nk, int D,
                          double scale, double *p) {
  double m = -INFINITY;
  for (int j = 0; j < nk; j++) {
    double s = 0.0;
    const double *kj = kbase + (int64_t)j * kstride;
    for (int c = 0; c < D; c++) s += q[c] * kj[c];
    s *= scale;
    p[j] = s;
    if (s > m) m = s;
  }
  double z = 0.0;
  for (int j = 0; j < nk; j++) {
    p[j] = exp(p[j] - m);
    z += p[j];
  }
  for (int j = 0; j < nk; j++) p[j] /= z;
  return m + log(z);
}

/* Keys attended in sequence i: all L, or the caller's count clamped to [0, L] (a count beyond
 * the sequence, like a negative one, is a statement about padding, not a request to read
 * past the end). */
static int attended_keys(const int32_t *seqused, int i, int L) {
  if (!seqused) return L;
  return seqused[i] < 0 ? 0 : seqused[i] > L ? L : seqused[i];
}

static int fwd_impl(const double *q, const double *k, const double *v, const int32_t *cu,
                    const int32_t *seqused, int B, int H, int D, double scale, const uint8_t *keep,
                    const int64_t *keep_off, double keep_scale, double *o, double *lse) {
  if (check_cu(cu, B) || H <= 0 || D <= 0) return 1;
  const int64_t T = cu[B];
  const int64_t ts = (int64_t)H * D; /* token stride */
  int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int i = 0; i < B; i++) {
    for (int h = 0; h < H; h++) {
      const int r0 = cu[i], L = cu[i + 1] - cu[i];
      const int nk = attended_keys(seqused, i, L);
      if (L == 0) continue;
      double *p = (double *)malloc(sizeof(double) * (size_t)(nk > 0 ? nk : 1));
      if (!p) {
        fail = 1;
        continue;
      }
      for (int r = 0; r < L; r++) {
        const double *qr = q + (r0 + r) * ts + (int64_t)h * D;
        double *orow = o + (r0 + r) * ts + (int64_t)h * D;
        if (nk <= 0) {
          for (int c = 0; c < D; c++) orow[c] = 0.0;
          if (lse) lse[(int64_t)h * T + r0 + r] = -INFINITY;
          continue;
        }
        double l = softmax_row(qr, k + r0 * ts + (int64_t)h * D, ts, nk, D, scale, p);
        for (int c = 0; c < D; c++) orow[c] = 0.0;
        for (int j = 0; j < nk; j++) {
          const double *vj = v + (r0 + j) * ts + (int64_t)h * D;
          double pj = p[j];
          if (keep) pj *= keep[keep_off[i] + ((int64_t)h * L + r) * L + j] ? keep_scale : 0.0;
          for (int c = 0; c < D; c++) orow[c] += pj * vj[c];
        }
        if (lse) lse[(int64_t)h * T + r0 + r] = l;
      }
      free(p);
    }
  }
  return fail;
}

int oracle_fmha_varlen_fwd(const double *q, const double *k, const double *v, const int32_t *cu,
                           const int32_t *seqused, int B, int H, int D, double scale, double *o,
                           double *lse) {
  return fwd_impl(q, k, v, cu, seqused, B, H, D, scale, NULL, NULL, 1.0, o, lse);
}

int oracle_fmha_varlen_fwd_dropout(const double *q, const double *k, const double *v,
                                   const int32_t *cu, const int32_t *seqused, int B, int H, int D,
                                   double scale, const uint8_t *keep, const int64_t *keep_off,
                                   double keep_scale, double *o, double *lse) {
  if (!keep || !keep_off) return 1;
  return fwd_impl(q, k, v, cu, seqused, B, H, D, scale, keep, keep_off, keep_scale, o, lse);
}

static int bwd_impl(const double *q, const double *k, const double *v, const double *dO,
                    const int32_t *cu, const int32_t *seqused, int B, int H, int D, double scale,
                    const uint8_t *keep, const int64_t *keep_off, double keep_scale, double *dq,
                    double *dk, double *dv) {
  if (check_cu(cu, B) || H <= 0 || D <= 0) return 1;
  const int64_t ts = (int64_t)H * D;
  int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int i = 0; i < B; i++) {
    for (int h = 0; h < H; h++) {
      const int r0 = cu[i], L = cu[i + 1] - cu[i];
      const int nk = attended_keys(seqused, i, L);
      if (L == 0) continue;
      const int64_t hb = (int64_t)h * D;
      double *p = (double *)malloc(sizeof(double) * (size_t)(2 * (nk > 0 ? nk : 1)));
      if (!p) {
        fail = 1;
        continue;
      }
      double *dp = p + (nk > 0 ? nk : 1);
      /* this (sequence, head) owns rows r0..r0+L-1 of dq, dk, dv exclusively */
      for (int r = 0; r < L; r++)
        for (int c = 0; c < D; c++) {
          dq[(r0 + r) * ts + hb + c] = 0.0;
          dk[(r0 + r) * ts + hb + c] = 0.0;
          dv[(r0 + r) * ts + hb + c] = 0.0;
        }
      for (int r = 0; r < L && nk > 0; r++) {
        const double *qr = q + (r0 + r) * ts + hb;
        const double *gr = dO + (r0 + r) * ts + hb;
        softmax_row(qr, k + r0 * ts + hb, ts, nk, D, scale, p);
        double Dr = 0.0;
        for (int j = 0; j < nk; j++) {
          const double *vj = v + (r0 + j) * ts + hb;
          double *dvj = dv + (r0 + j) * ts + hb;
          double t = 0.0;
          /* M c of this element; 1 without dropout */
          const double mc =
              keep ? (keep[keep_off[i] + ((int64_t)h * L + r) * L + j] ? keep_scale : 0.0) : 1.0;
          for (int c = 0; c < D; c++) {
            dvj[c] += p[j] * mc * gr[c]; /* dV = (P o M c)^T dO */
            t += gr[c] * vj[c];          /* dO V^T */
          }
          dp[j] = t * mc; /* dP = (dO V^T) o M c */
          Dr += p[j] * dp[j];
        }
        double *dqr = dq + (r0 + r) * ts + hb;
        for (int j = 0; j < nk; j++) {
          const double ds = p[j] * (dp[j] - Dr);
          const double *kj = k + (r0 + j) * ts + hb;
          double *dkj = dk + (r0 + j) * ts + hb;
          for (int c = 0; c < D; c++) {
            dqr[c] += scale * ds * kj[c];
            dkj[c] += scale * ds * qr[c];
          }
        }
      }
      free(p);
    }
  }
  return fail;
}

int oracle_fmha_varlen_bwd(const double *q, const double *k, const double *v, const double *dO,
                           const int32_t *cu, const int32_t *seqused, int B, int H, int D,
                           double scale, double *dq, double *dk, double *dv) {
  return bwd_impl(q, k, v, dO, cu, seqused, B, H, D, scale, NULL, NULL, 1.0, dq, dk, dv);
}

int oracle_fmha_varlen_bwd_dropout(const double *q, const double *k, const double *v,
                                   const double *dO, const int32_t *cu, const int32_t *seqused,
                                   int B, int H, int D, double scale, const uint8_t *keep,
                                   const int64_t *keep_off, double keep_scale, double *dq,
                                   double *dk, double *dv) {
  if (!keep || !keep_off) return 1;
  return bwd_impl(q, k, v, dO, cu, seqused, B, H, D, scale, keep, keep_off, keep_scale, dq, dk, dv);
}

int oracle_num_threads(void) {
  int n = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp single
    n = omp_get_num_threads();
  }
#endif
  return n;
}
