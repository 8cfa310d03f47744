/*
 * hca_plain_oracle.c: the plain definitions, in fp64, of the three quantities that the
 * other oracle files evaluate in a bit-reproducible (integer or fixed-order fp32) form.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path links, loads or calls this file,
 * and it shares no code, table or constant with the HIP library.  It uses hco_h2f of
 * hca_oracle.c (the fp16 decode) and nothing else.
 *
 * Why it exists: a bit-exact comparison needs arithmetic that a second implementation can
 * reproduce, so hco_score maps the query to fixed point, hco_vq_score adds table entries on
 * a power-of-two grid and hco_topp turns weights into integers.  Those are readings.  The
 * functions below are what the paper writes, with no such device, so that tests can bound
 * the distance between each reading and the definition it stands for:
 *
 *   hco_score_plain      z~ = q . Q(K)^T of Eq. 2 (Sec. 3.2) with the query as it is:
 *                        z[hq][j] = sum_c q_c * (scale_g * code_c + zero_g), every term fp64
 *   hco_score_fp32       the same in plain fp32 arithmetic with the unquantised query (ascending fused
 *                        multiply-add chains per group), for the distance to the fixed-point form
 *   hco_vq_score_plain   Eq. 3: z[hq][j] = sum_i T[hq][i][P[j][i]], fp64 sum of the fp32 table
 *   hco_topp_plain       Eq. 4: a = softmax(sel * sm_scale) over the row in fp64; slots sorted by
 *                        (sel descending, slot ascending); k* = the least k whose sorted prefix
 *                        sums to >= tau.  Also returns the sorted order and the running sums, so
 *                        that a test can read the mass of any prefix.
 *
 * Parity status: these are definitions, pinned in tests against numpy on small inputs; the
 * per-KV-head reading of Eq. 4's weights (softmax of the selection score) is this build's and
 * "parity unpinned" by the paper.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#define HCO_OK 0
#define HCO_ERR_BAD_ARG (-1)
#define HCO_ERR_NAN (-2)

float hco_h2f(uint16_t h);   /* hca_oracle.c */

/* q [R*G][D] fp16; codes [R][cap][D*bits/8] (channel c in bits [(c*bits)%8, +bits) of byte c*bits/8);
 * scale, zero [R][cap][D/gs] fp16; z [R*G][cap] fp64, written for j < n[r]. */
int hco_score_plain(const uint16_t* q, const uint8_t* codes, const uint16_t* scale, const uint16_t* zero,
                    int64_t R, int G, int D, int bits, int gs, int64_t cap, const int64_t* n, double* z) {
  if (D <= 0 || gs <= 0 || D % gs != 0 || (bits != 2 && bits != 4 && bits != 8) || G < 1) return HCO_ERR_BAD_ARG;
  const int NG = D / gs, CB = D * bits / 8;
  for (int64_t hq = 0; hq < R * G; ++hq) {
    int64_t r = hq / G;
    for (int64_t j = 0; j < n[r]; ++j) {
      const uint8_t* crow = codes + (r * cap + j) * CB;
      double s = 0.0;
      for (int c = 0; c < D; ++c) {
        int bit = c * bits;
        int code = (crow[bit >> 3] >> (bit & 7)) & ((1 << bits) - 1);
        double khat = (double)hco_h2f(scale[(r * cap + j) * NG + c / gs]) * (double)code
                      + (double)hco_h2f(zero[(r * cap + j) * NG + c / gs]);
        s += (double)hco_h2f(q[hq * D + c]) * khat;
      }
      z[hq * cap + j] = s;
    }
  }
  return HCO_OK;
}

/* The same score in plain fp32 with the query as it is (no fixed point), the form one would write first:
 * per group D_g = fused multiply-add chain over the group's channels in ascending order of q_c * code_c from
 * 0.0f; Q_g = fp32 sum of q_c in ascending order; t_g = fmaf(scale_g, D_g, zero_g * Q_g);
 * z = (t0 + t1) + (t2 + t3) (two groups: t0 + t1; otherwise left to right).  Not reproducible bit for bit on
 * a matrix core (the chain's order is), which is why hco_score uses the fixed-point query; a test bounds the
 * distance between the two.  z [R*G][cap] fp32, written for j < n[r]. */
int hco_score_fp32(const uint16_t* q, const uint8_t* codes, const uint16_t* scale, const uint16_t* zero,
                   int64_t R, int G, int D, int bits, int gs, int64_t cap, const int64_t* n, float* z) {
  if (D <= 0 || gs <= 0 || D % gs != 0 || (bits != 2 && bits != 4 && bits != 8) || G < 1) return HCO_ERR_BAD_ARG;
  const int NG = D / gs, CB = D * bits / 8;
  if (NG > 16) return HCO_ERR_BAD_ARG;
  for (int64_t hq = 0; hq < R * G; ++hq) {
    int64_t r = hq / G;
    float Qg[16];
    for (int g = 0; g < NG; ++g) {
      float acc = 0.0f;
      for (int c = g * gs; c < (g + 1) * gs; ++c) acc = acc + hco_h2f(q[hq * D + c]);
      Qg[g] = acc;
    }
    for (int64_t j = 0; j < n[r]; ++j) {
      const uint8_t* crow = codes + (r * cap + j) * CB;
      float t[16];
      for (int g = 0; g < NG; ++g) {
        float Dg = 0.0f;
        for (int c = g * gs; c < (g + 1) * gs; ++c) {
          int bit = c * bits;
          int code = (crow[bit >> 3] >> (bit & 7)) & ((1 << bits) - 1);
          Dg = fmaf(hco_h2f(q[hq * D + c]), (float)code, Dg);
        }
        float zq = hco_h2f(zero[(r * cap + j) * NG + g]) * Qg[g];
        t[g] = fmaf(hco_h2f(scale[(r * cap + j) * NG + g]), Dg, zq);
      }
      float s;
      if (NG == 4) { float a = t[0] + t[1], b = t[2] + t[3]; s = a + b; }
      else { s = t[0]; for (int g = 1; g < NG; ++g) s = s + t[g]; }
      z[hq * cap + j] = s;
    }
  }
  return HCO_OK;
}

/* T [R*G][g][c] fp32; P [R][cap][g] uint16; z [R*G][cap] fp64, written for j < n[r]. */
int hco_vq_score_plain(const float* T, const uint16_t* P, int64_t R, int G, int g, int c, int64_t cap,
                       const int64_t* n, double* z) {
  if (G < 1 || g < 1 || c < 1) return HCO_ERR_BAD_ARG;
  for (int64_t hq = 0; hq < R * G; ++hq) {
    int64_t r = hq / G;
    for (int64_t j = 0; j < n[r]; ++j) {
      double s = 0.0;
      for (int i = 0; i < g; ++i) {
        int p = P[(r * cap + j) * g + i];
        if (p >= c) return HCO_ERR_BAD_ARG;
        s += (double)T[(hq * g + i) * c + p];
      }
      z[hq * cap + j] = s;
    }
  }
  return HCO_OK;
}

typedef struct { float v; int32_t i; } pl_pair;

static int pl_cmp(const void* a, const void* b) {
  const pl_pair* x = (const pl_pair*)a; const pl_pair* y = (const pl_pair*)b;
  if (x->v > y->v) return -1;
  if (x->v < y->v) return 1;
  return (x->i > y->i) - (x->i < y->i);
}

/* sel [R][cap] fp32; kstar [R]; order_opt [R][cap] int32 (the row's slots in sorted order) or NULL;
 * cum_opt [R][cap] fp64 (cum[t] = a_(1) + ... + a_(t+1), summed in sorted order) or NULL. */
int hco_topp_plain(const float* sel, int64_t R, int64_t cap, const int64_t* n, double sm_scale, double tau,
                   int64_t* kstar, int32_t* order_opt, double* cum_opt) {
  if (!(tau > 0.0) || !(sm_scale > 0.0)) return HCO_ERR_BAD_ARG;
  int err = 0;
  for (int64_t r = 0; r < R; ++r) {
    int64_t nr = n[r];
    kstar[r] = 0;
    if (nr <= 0) continue;
    pl_pair* p = (pl_pair*)malloc(sizeof(pl_pair) * (size_t)nr);
    double* a = (double*)malloc(sizeof(double) * (size_t)nr);
    for (int64_t j = 0; j < nr; ++j) {
      p[j].v = sel[r * cap + j]; p[j].i = (int32_t)j;
      if (isnan(p[j].v)) err = 1;
    }
    qsort(p, (size_t)nr, sizeof(pl_pair), pl_cmp);
    double m = (double)p[0].v * sm_scale, Z = 0.0;
    for (int64_t j = 0; j < nr; ++j) { a[j] = exp((double)p[j].v * sm_scale - m); Z += a[j]; }
    double run = 0.0;
    int64_t ks = nr;
    int found = 0;
    for (int64_t j = 0; j < nr; ++j) {
      run += a[j] / Z;
      if (cum_opt) cum_opt[r * cap + j] = run;
      if (order_opt) order_opt[r * cap + j] = p[j].i;
      if (!found && run >= tau) { ks = j + 1; found = 1; }
    }
    kstar[r] = ks;
    free(p); free(a);
  }
  return err ? HCO_ERR_NAN : HCO_OK;
}
