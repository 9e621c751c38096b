/* Runs the fp64 oracle (compiled together with this file, both under
 * -fsanitize=address,undefined) over ragged batches and re-checks invariants that hold
 * whatever the inputs are:
 *   - a sequence of one token has O = V and zero dQ, dK;
 *   - softmax rows sum to one, so sum_j dV_j = sum_r dO_r over a sequence;
 *   - rows of dS sum to zero, so sum_j dK_j = 0 over a sequence;
 *   - sequences with no attended key give O = 0, LSE = -inf and zero gradients.
 * Any out-of-bounds access or undefined operation inside the oracle ends the run. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_fmha_varlen_fwd(const double *q, const double *k, const double *v, const int32_t *cu,
                           const int32_t *seqused, int B, int H, int D, double scale, double *o,
                           double *lse);
int oracle_fmha_varlen_bwd(const double *q, const double *k, const double *v, const double *dO,
                           const int32_t *cu, const int32_t *seqused, int B, int H, int D,
                           double scale, double *dq, double *dk, double *dv);

static uint64_t state = 0x2208081240ull;
static double rnd(void) {
  state = state * 6364136223846793005ull + 1442695040888963407ull;
  return (double)((state >> 11) & 0xfffff) / (double)0x100000 * 2.0 - 1.0;
}

#define CHECK(c)                                                        \
  do {                                                                  \
    if (!(c)) {                                                         \
      fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #c); \
      return 1;                                                         \
    }                                                                   \
  } while (0)

static int one_case(const int *len, const int *used, int B, int H) {
  const int D = 64;
  int32_t *cu = malloc(sizeof(int32_t) * (size_t)(B + 1));
  int32_t *su = used ? malloc(sizeof(int32_t) * (size_t)B) : NULL;
  cu[0] = 0;
  for (int i = 0; i < B; i++) {
    cu[i + 1] = cu[i] + len[i];
    if (su) su[i] = used[i];
  }
  const size_t T = (size_t)cu[B], n = T * (size_t)H * D;
  double *buf = malloc(sizeof(double) * (n * 8 + 1));
  double *q = buf, *k = buf + n, *v = buf + 2 * n, *g = buf + 3 * n, *o = buf + 4 * n, *dq = buf + 5 * n,
         *dk = buf + 6 * n, *dv = buf + 7 * n;
  double *lse = malloc(sizeof(double) * (T * (size_t)H + 1));
  for (size_t i = 0; i < 4 * n; i++) buf[i] = rnd();
  CHECK(oracle_fmha_varlen_fwd(q, k, v, cu, su, B, H, D, 0.125, o, lse) == 0);
  CHECK(oracle_fmha_varlen_bwd(q, k, v, g, cu, su, B, H, D, 0.125, dq, dk, dv) == 0);
  for (int i = 0; i < B; i++) {
    const int L = len[i], nk = su ? (su[i] < 0 ? 0 : su[i] > L ? L : su[i]) : L;
    for (int h = 0; h < H; h++)
      for (int c = 0; c < D; c++) {
        double sum_dv = 0, sum_do = 0, sum_dk = 0;
        for (int r = 0; r < L; r++) {
          const size_t at = ((size_t)(cu[i] + r) * H + h) * D + c;
          CHECK(isfinite(o[at]) && isfinite(dq[at]) && isfinite(dk[at]) && isfinite(dv[at]));
          sum_dv += dv[at];
          sum_do += g[at];
          sum_dk += dk[at];
          if (nk == 0) CHECK(o[at] == 0 && dq[at] == 0 && dk[at] == 0 && dv[at] == 0);
          if (L == 1 && nk == 1) CHECK(fabs(o[at] - v[at]) < 1e-12 && fabs(dq[at]) < 1e-12 && fabs(dk[at]) < 1e-12);
        }
        if (nk > 0) CHECK(fabs(sum_dv - sum_do) < 1e-9 * (1 + L) && fabs(sum_dk) < 1e-9 * (1 + L));
      }
    for (int h = 0; h < H; h++)
      for (int r = 0; r < L; r++) {
        const double l = lse[(size_t)h * T + (size_t)(cu[i] + r)];
        CHECK(nk == 0 ? (isinf(l) && l < 0) : isfinite(l));
      }
  }
  free(lse);
  free(buf);
  free(su);
  free(cu);
  return 0;
}

int main(void) {
  const int a[] = {1, 3, 0, 17, 64, 65}, b[] = {130, 1, 1}, c[] = {5, 40, 7, 33};
  const int cu_used[] = {0, -2, 7, 40};
  if (one_case(a, NULL, 6, 2) || one_case(b, NULL, 3, 1) || one_case(c, cu_used + 0, 4, 3)) return 1;
  /* a decreasing prefix sum is refused, not followed */
  int32_t bad[] = {0, 5, 3};
  double x[5 * 64] = {0};
  if (oracle_fmha_varlen_fwd(x, x, x, bad, NULL, 2, 1, 64, 1.0, x, x) == 0) {
    fprintf(stderr, "decreasing cu_seqlens accepted\n");
    return 1;
  }
  puts("oracle under sanitizers: ok");
  return 0;
}
