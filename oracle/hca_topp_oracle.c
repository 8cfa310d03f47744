/*
 * hca_topp_oracle.c: slow, plain CPU reference for the paper's own selection rule
 * (Sec. 3.2, Eq. 4): sort the approximate attention weights in descending order and keep
 * the shortest prefix whose cumulative weight reaches the threshold tau.
 *
 * TEST INFRASTRUCTURE ONLY (parity oracle of hca_topp); shares no code with the HIP library.
 *
 * The weights are those of the row's selection scores: a~_j = softmax_j(sel_j * sm_scale)
 * over the resident slots of a (sequence, KV head) row, sel being the per-KV-head score the
 * scan leaves (the maximum over the KV head's query heads).  k* is an integer decided by a
 * floating-point sum, so the sum is made exact: every weight is turned into an integer by
 * one fixed sequence of single fp32 operations and the cumulative test runs on integers,
 * which no summation order can change.
 *
 *   l_j = sel_j * sm_scale                    (fp32)
 *   m   = max_j l_j,  u_j = l_j - m           (fp32, u_j <= 0)
 *   w_j = W(u_j): t = u * 1.44269504f; t < -64 -> 0; fl = floorf(t); f = t - fl (exact, in [0, 1));
 *         p = c0 + f (c1 + f (c2 + ... f c6)) by fmaf, c_k = (ln 2)^k / k! (2^f to ~1e-5);
 *         mant = (uint64) (p * 2^31)  (truncation);  w = mant >> (int)(-fl)
 *         so w ~ exp(u) * 2^31, at most 2^32, zero below exp(u) ~ 2^-32
 *   Z = sum_j w_j                              (uint64, exact)
 *   Theta = max(1, floor(Z * tau_fix / 2^64)), tau_fix = floor(tau * 2^64) for tau < 1; Theta = Z for tau >= 1
 *   order: sel descending, slot ascending (-0 == +0), as in hco_topk
 *   k* = the least k with  w_(1) + ... + w_(k) >= Theta,  then clipped to k_max
 * Output as hco_topk: the k* slots in ascending order, -1 padded.
 *
 * Parity status: Eq. 4 itself is the paper's; taking the weights from the per-KV-head selection
 * score, the integer weight function and the clip are readings of this build ("parity
 * unpinned" by the paper), pinned against an fp64 softmax, closed forms and brute force.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#define HCO_OK 0
#define HCO_ERR_BAD_ARG (-1)
#define HCO_ERR_NAN (-2)

/* the integer weight W(u) of a logit u <= 0 relative to the row maximum */
uint64_t hco_topp_weight(float u) {
  float t = u * 1.44269504f;
  if (!(t >= -64.0f)) return 0;                 /* also -inf and NaN */
  float fl = floorf(t);
  float f = t - fl;
  float p = 1.5403530e-4f;
  p = fmaf(p, f, 1.3333558e-3f);
  p = fmaf(p, f, 9.6181291e-3f);
  p = fmaf(p, f, 5.5504109e-2f);
  p = fmaf(p, f, 2.4022651e-1f);
  p = fmaf(p, f, 6.9314718e-1f);
  p = fmaf(p, f, 1.0f);
  uint64_t mant = (uint64_t)(p * 2147483648.0f);
  int sh = (int)(-fl);
  return sh >= 64 ? 0 : mant >> sh;
}

typedef struct { float v; int32_t i; } tp_pair;

static int tp_cmp(const void* a, const void* b) {
  const tp_pair* x = (const tp_pair*)a; const tp_pair* y = (const tp_pair*)b;
  if (x->v > y->v) return -1;
  if (x->v < y->v) return 1;
  return (x->i > y->i) - (x->i < y->i);
}
static int tp_cmp_int(const void* a, const void* b) {
  int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return (x > y) - (x < y);
}

/* sel [R][cap]; idx [R][k_max] (-1 padded); count [R] = min(k*, k_max); kstar_opt [R] = the unclipped k*;
 * mass_opt [R][2] = (Theta, Z). */
int hco_topp(const float* sel, int64_t R, int64_t cap, const int64_t* n, float sm_scale, double tau,
             int64_t k_max, int32_t* idx, int32_t* count, int64_t* kstar_opt, uint64_t* mass_opt) {
  if (k_max < 0 || !(tau > 0.0) || !(sm_scale > 0.0f)) return HCO_ERR_BAD_ARG;
  int err = 0;
  for (int64_t r = 0; r < R; ++r) {
    int64_t nr = n[r];
    int32_t* out = idx + r * k_max;
    for (int64_t j = 0; j < k_max; ++j) out[j] = -1;
    count[r] = 0;
    if (kstar_opt) kstar_opt[r] = 0;
    if (mass_opt) { mass_opt[2 * r] = 0; mass_opt[2 * r + 1] = 0; }
    if (nr <= 0) continue;
    tp_pair* p = (tp_pair*)malloc(sizeof(tp_pair) * (size_t)nr);
    float m = -INFINITY;
    for (int64_t j = 0; j < nr; ++j) {
      float v = sel[r * cap + j];
      if (isnan(v)) err = 1;
      p[j].v = v; p[j].i = (int32_t)j;
      float l = v * sm_scale;
      if (l > m) m = l;
    }
    qsort(p, (size_t)nr, sizeof(tp_pair), tp_cmp);
    uint64_t Z = 0;
    for (int64_t j = 0; j < nr; ++j) Z += hco_topp_weight(p[j].v * sm_scale - m);
    uint64_t theta;
    if (tau >= 1.0) {
      theta = Z;
    } else {
      uint64_t tau_fix = (uint64_t)ldexp(tau, 64);
      theta = (uint64_t)(((unsigned __int128)Z * tau_fix) >> 64);
      if (theta < 1) theta = 1;
    }
    uint64_t run = 0;
    int64_t ks = nr;
    for (int64_t j = 0; j < nr; ++j) {
      run += hco_topp_weight(p[j].v * sm_scale - m);
      if (run >= theta) { ks = j + 1; break; }
    }
    int64_t kk = ks < k_max ? ks : k_max;
    for (int64_t j = 0; j < kk; ++j) out[j] = p[j].i;
    qsort(out, (size_t)kk, sizeof(int32_t), tp_cmp_int);
    count[r] = (int32_t)kk;
    if (kstar_opt) kstar_opt[r] = ks;
    if (mass_opt) { mass_opt[2 * r] = theta; mass_opt[2 * r + 1] = Z; }
    free(p);
  }
  return err ? HCO_ERR_NAN : HCO_OK;
}
