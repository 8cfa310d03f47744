/*
 * hca_oracle.c: slow, plain CPU reference for the HCAttention decode path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the parity oracle and the timed CPU
 * baseline.  Nothing in the product path links, loads or calls it, and it
 * shares no code, header, table or helper with the HIP library.
 *
 * What it computes, with the passage of the paper each function follows:
 *   hco_attention_exact   standard attention, Eq. 1 (Sec. 3.2)
 *   hco_quantize          the key compressor Q(K) of Eq. 2, in the per-token
 *                         asymmetric uniform form (b-bit codes, one fp16 scale
 *                         and zero per channel group)
 *   hco_dequantize        the inverse map, k_hat = scale * code + zero
 *   hco_query_fixed       15-bit fixed-point image of the query
 *   hco_score             z~ = q . Q(K)^T of Eq. 2 / Eq. 3, evaluated group by
 *                         group, plus the per-KV-head selection score
 *   hco_topk              the sorted prefix Pi_k of Sec. 3.2 ("sort in
 *                         descending order"), with k given instead of derived
 *                         from tau (Eq. 4)
 *   hco_lse               log of the softmax denominator over all resident tokens
 *                         (Sec. 3.2), per query head
 *   hco_attend            softmax over the selected set and the weighted value
 *                         sum of Eq. 5 (optionally with the paper's own weights,
 *                         normalised over all tokens); accumulated-score update
 *   hco_evict             keep-M by accumulated score with stable compaction
 *
 * Precision.  Everything that feeds an integer decision (codes, the selection
 * score, the top-k order) is single IEEE fp32 operations in one fixed order so
 * that a second implementation can reproduce the bits; the file must be
 * compiled with -ffp-contract=off and without fast-math.  Softmax and the
 * weighted sum accumulate in fp64.
 *
 * Parity status.  The quantiser form (scale/zero) and the accumulated-score
 * eviction policy are choices of this build, not of the paper: they are pinned
 * by invariants, closed forms and brute force only ("parity unpinned" by the
 * paper itself).  Scores, selection and the weighted sum are pinned against
 * Eq. 1 evaluated in fp64 and against library sort / softmax routines.
 *
 * Canonical (oracle-side) cache layout for R = batch * kv_heads rows:
 *   codes [R][cap][D*bits/8]  channel c lives in bits [(c*bits)%8, +bits) of
 *                             byte floor(c*bits/8)
 *   scale [R][cap][D/gs]      fp16 bit patterns
 *   zero  [R][cap][D/gs]      fp16 bit patterns
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define HCO_OK 0
#define HCO_ERR_BAD_ARG (-1)
#define HCO_ERR_NAN (-2)

/* ---------------------------------------------------------------- fp16 --- */

/* IEEE binary16 bit pattern -> fp32 (exact). */
float hco_h2f(uint16_t h) {
  int sign = (h >> 15) & 1;
  int e = (h >> 10) & 31;
  int m = h & 1023;
  float v;
  if (e == 0) {
    v = ldexpf((float)m, -24);            /* zero and subnormals */
  } else if (e == 31) {
    v = m ? NAN : INFINITY;
  } else {
    v = ldexpf((float)(1024 + m), e - 25); /* 1.m * 2^(e-15) */
  }
  return sign ? -v : v;
}

/* fp32 -> IEEE binary16 bit pattern, round to nearest, ties to even. */
uint16_t hco_f2h(float f) {
  uint16_t sign = signbit(f) ? 0x8000u : 0u;
  float x = fabsf(f);
  if (isnan(x)) return (uint16_t)(sign | 0x7e00u);
  if (x >= 65520.0f) return (uint16_t)(sign | 0x7c00u); /* halfway to 2^16 rounds to inf */
  if (x < 6.103515625e-05f) {                           /* below 2^-14: subnormal grid 2^-24 */
    int m = (int)rintf(ldexpf(x, 24));                  /* exact product, one rounding */
    return (uint16_t)(sign | (uint16_t)m);              /* m == 1024 is the smallest normal */
  }
  int e = ilogbf(x);
  int m = (int)rintf(ldexpf(x, 10 - e));                /* in [1024, 2048] */
  if (m == 2048) { m = 1024; e += 1; }
  return (uint16_t)(sign | (uint16_t)((e + 15) << 10) | (uint16_t)(m - 1024));
}

int hco_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

static int shape_ok(int D, int bits, int gs) {
  if (!(bits == 2 || bits == 4 || bits == 8)) return 0;
  if (!(gs == 32 || gs == 64)) return 0;
  if (D <= 0 || D > 512 || D % gs != 0) return 0;
  return 1;
}

static inline int get_code(const uint8_t* row, int c, int bits) {
  int bit = c * bits;
  return (row[bit >> 3] >> (bit & 7)) & ((1 << bits) - 1);
}

/* ------------------------------------------------------- Eq. 1, exact --- */

/* y = softmax(q K^T * sm_scale) V for one head, all in fp64 from fp16 inputs.
 * K, V: [n][D] fp16 bits.  Follows Eq. 1 term by term. */
int hco_attention_exact(const uint16_t* q, const uint16_t* K, const uint16_t* V,
                        int64_t n, int D, double sm_scale, double* y) {
  if (n <= 0 || D <= 0) return HCO_ERR_BAD_ARG;
  double* z = (double*)malloc(sizeof(double) * (size_t)n);
  if (!z) return HCO_ERR_BAD_ARG;
  double m = -INFINITY;
  for (int64_t j = 0; j < n; ++j) {
    double s = 0.0;
    for (int c = 0; c < D; ++c) s += (double)hco_h2f(q[c]) * (double)hco_h2f(K[j * D + c]);
    z[j] = s * sm_scale;
    if (z[j] > m) m = z[j];
  }
  double Z = 0.0;
  for (int64_t j = 0; j < n; ++j) { z[j] = exp(z[j] - m); Z += z[j]; }
  for (int c = 0; c < D; ++c) y[c] = 0.0;
  for (int64_t j = 0; j < n; ++j) {
    double a = z[j] / Z;
    for (int c = 0; c < D; ++c) y[c] += a * (double)hco_h2f(V[j * D + c]);
  }
  free(z);
  return HCO_OK;
}

/* ---------------------------------------------------------- quantise --- */

/* Quantise T new tokens per row and append them at slot n0[r].
 * k_new: [R][T][D] fp16 bits.  Per (token, group):
 *   mn = min x, mx = max x (fp32 images of the fp16 inputs, -0 stored as +0)
 *   scale = fp16_rne((mx - mn) / qmax), replaced by 1.0 when it rounds to 0
 *   inv   = 1.0f / (float)scale
 *   code  = clamp(rint((x - mn) * inv), 0, qmax)        (ties to even)
 *   zero  = fp16(mn)                                     (exact)
 */
int hco_quantize(const uint16_t* k_new, int64_t R, int64_t T, int D, int bits, int gs,
                 int64_t cap, const int64_t* n0,
                 uint8_t* codes, uint16_t* scale, uint16_t* zero) {
  if (!shape_ok(D, bits, gs) || R < 0 || T < 0) return HCO_ERR_BAD_ARG;
  const int NG = D / gs, CB = D * bits / 8, qmax = (1 << bits) - 1;
  for (int64_t r = 0; r < R; ++r)
    if (n0[r] < 0 || n0[r] + T > cap) return HCO_ERR_BAD_ARG;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < R; ++r) {
    for (int64_t t = 0; t < T; ++t) {
      const uint16_t* x16 = k_new + (r * T + t) * D;
      int64_t slot = n0[r] + t;
      uint8_t* crow = codes + (r * cap + slot) * CB;
      memset(crow, 0, (size_t)CB);
      for (int g = 0; g < NG; ++g) {
        float mn = INFINITY, mx = -INFINITY;
        for (int c = g * gs; c < (g + 1) * gs; ++c) {
          float x = hco_h2f(x16[c]);
          if (x < mn) mn = x;
          if (x > mx) mx = x;
        }
        if (mn == 0.0f) mn = 0.0f;              /* canonical +0 */
        float range = mx - mn;
        uint16_t sh = hco_f2h(range / (float)qmax);
        if ((sh & 0x7fffu) == 0) sh = 0x3c00u;  /* 1.0 */
        float sc = hco_h2f(sh);
        float inv = 1.0f / sc;
        for (int c = g * gs; c < (g + 1) * gs; ++c) {
          float x = hco_h2f(x16[c]);
          float v = rintf((x - mn) * inv);
          if (v < 0.0f) v = 0.0f;
          if (v > (float)qmax) v = (float)qmax;
          int code = (int)v;
          int bit = c * bits;
          crow[bit >> 3] |= (uint8_t)(code << (bit & 7));
        }
        scale[(r * cap + slot) * NG + g] = sh;
        zero[(r * cap + slot) * NG + g] = hco_f2h(mn);
      }
    }
  }
  return HCO_OK;
}

/* k_hat[r][j][c] = fma(scale, code, zero) for slots j < n[r]; out: [R][cap][D] fp32 */
int hco_dequantize(const uint8_t* codes, const uint16_t* scale, const uint16_t* zero,
                   int64_t R, int D, int bits, int gs, int64_t cap, const int64_t* n,
                   float* khat) {
  if (!shape_ok(D, bits, gs)) return HCO_ERR_BAD_ARG;
  const int NG = D / gs, CB = D * bits / 8;
  for (int64_t r = 0; r < R; ++r)
    for (int64_t j = 0; j < n[r]; ++j)
      for (int c = 0; c < D; ++c) {
        int g = c / gs;
        float sc = hco_h2f(scale[(r * cap + j) * NG + g]);
        float zr = hco_h2f(zero[(r * cap + j) * NG + g]);
        khat[(r * cap + j) * D + c] =
            fmaf(sc, (float)get_code(codes + (r * cap + j) * CB, c, bits), zr);
      }
  return HCO_OK;
}

/* ------------------------------------------------------------- score --- */

/* Fixed-point image of one query head: qfx[c] = rint(q[c] * 2^s) with
 * s = 13 - floor(log2(max|q|)), so that |qfx| < 2^14 (s = 0 for a zero query). */
int hco_query_fixed(const uint16_t* q, int D, int32_t* qfx, int32_t* s_out) {
  float amax = 0.0f;
  for (int c = 0; c < D; ++c) {
    float a = fabsf(hco_h2f(q[c]));
    if (isnan(a) || isinf(a)) return HCO_ERR_NAN;
    if (a > amax) amax = a;
  }
  int s = (amax == 0.0f) ? 0 : 13 - ilogbf(amax);
  for (int c = 0; c < D; ++c) qfx[c] = (int32_t)rintf(ldexpf(hco_h2f(q[c]), s));
  *s_out = s;
  return HCO_OK;
}

/* z~ of one (query head, token): per group gamma
 *     D_g = sum_c qfx[c]*code[c]   (exact, int32)
 *     Q_g = sum_c qfx[c]           (exact, int32)
 *     t_g = fma(scale_g, (float)D_g, zero_g * (float)Q_g)
 * then (t0+t1)+(t2+t3) (or t0+t1, or t0), times 2^-s.  D must give 1, 2 or 4 groups. */
static float score_one(const int32_t* qfx, int s, const uint8_t* crow, const uint16_t* sc,
                       const uint16_t* zr, int D, int bits, int gs) {
  const int NG = D / gs;
  float t[4] = {0, 0, 0, 0};
  for (int g = 0; g < NG; ++g) {
    int32_t Dg = 0, Qg = 0;
    for (int c = g * gs; c < (g + 1) * gs; ++c) {
      Dg += qfx[c] * get_code(crow, c, bits);
      Qg += qfx[c];
    }
    float zq = hco_h2f(zr[g]) * (float)Qg;
    t[g] = fmaf(hco_h2f(sc[g]), (float)Dg, zq);
  }
  float sum;
  if (NG == 4) { float a = t[0] + t[1]; float b = t[2] + t[3]; sum = a + b; }
  else if (NG == 2) sum = t[0] + t[1];
  else sum = t[0];
  return ldexpf(sum, -s);
}

/* q: [R*G][D] fp16 (query head r*G+g uses row r); z: [R*G][cap] fp32 or NULL;
 * sel: [R][cap] fp32 = max over the G heads of a row. */
int hco_score(const uint16_t* q, const uint8_t* codes, const uint16_t* scale,
              const uint16_t* zero, int64_t R, int G, int D, int bits, int gs,
              int64_t cap, const int64_t* n, float* sel, float* z) {
  if (!shape_ok(D, bits, gs) || G <= 0 || G > 16) return HCO_ERR_BAD_ARG;
  const int NG = D / gs, CB = D * bits / 8;
  if (NG != 1 && NG != 2 && NG != 4) return HCO_ERR_BAD_ARG;
  int err = 0;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < R; ++r) {
    int32_t* qfx = (int32_t*)malloc(sizeof(int32_t) * (size_t)(G * D));
    int32_t s[16];
    for (int g = 0; g < G; ++g)
      if (hco_query_fixed(q + (r * G + g) * D, D, qfx + g * D, &s[g]) != HCO_OK) err = 1;
    for (int64_t j = 0; j < n[r]; ++j) {
      float best = -INFINITY;
      for (int g = 0; g < G; ++g) {
        float v = score_one(qfx + g * D, s[g], codes + (r * cap + j) * CB,
                            scale + (r * cap + j) * NG, zero + (r * cap + j) * NG, D, bits, gs);
        if (z) z[(r * G + g) * cap + j] = v;
        if (v > best) best = v;
      }
      sel[r * cap + j] = best;
    }
    free(qfx);
  }
  return err ? HCO_ERR_NAN : HCO_OK;
}

/* Softmax denominator over ALL resident tokens, per query head (Sec. 3.2: a~ = softmax(z~ / sqrt(d)) is
 * taken over the whole sequence before anything is selected):
 *   lse[hq] = log sum_{j < n} exp(z[hq][j] * sm_scale)      (fp32 product, fp64 exp / sum / log, cast to fp32)
 * z: [R*G][cap] as written by hco_score; rows without resident tokens give -inf. */
int hco_lse(const float* z, int64_t R, int G, int64_t cap, const int64_t* n, float sm_scale, float* lse) {
  if (G < 1 || G > 16) return HCO_ERR_BAD_ARG;
  for (int64_t hq = 0; hq < R * G; ++hq) {
    int64_t nr = n[hq / G];
    float m = -INFINITY;
    for (int64_t j = 0; j < nr; ++j) {
      float l = z[hq * cap + j] * sm_scale;
      if (l > m) m = l;
    }
    double acc = 0.0;
    for (int64_t j = 0; j < nr; ++j) acc += exp((double)(z[hq * cap + j] * sm_scale) - (double)m);
    lse[hq] = nr > 0 ? (float)((double)m + log(acc)) : -INFINITY;
  }
  return HCO_OK;
}

/* -------------------------------------------------------------- top-k --- */

typedef struct { float v; int32_t i; } hco_pair;

static int cmp_desc_then_index(const void* a, const void* b) {
  const hco_pair* x = (const hco_pair*)a; const hco_pair* y = (const hco_pair*)b;
  if (x->v > y->v) return -1;
  if (x->v < y->v) return 1;       /* -0 and +0 compare equal here */
  return (x->i > y->i) - (x->i < y->i);
}
static int cmp_int(const void* a, const void* b) {
  int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return (x > y) - (x < y);
}

/* Order slots [0, n) by (value descending, index ascending), keep the first
 * min(k, n), return them in ascending index order.  out: [k'] */
static int topk_row(const float* v, int64_t n, int64_t k, int32_t* out) {
  if (n <= 0 || k <= 0) return 0;
  hco_pair* p = (hco_pair*)malloc(sizeof(hco_pair) * (size_t)n);
  for (int64_t j = 0; j < n; ++j) { p[j].v = v[j]; p[j].i = (int32_t)j; }
  qsort(p, (size_t)n, sizeof(hco_pair), cmp_desc_then_index);
  int64_t kk = k < n ? k : n;
  for (int64_t j = 0; j < kk; ++j) out[j] = p[j].i;
  qsort(out, (size_t)kk, sizeof(int32_t), cmp_int);
  free(p);
  return (int)kk;
}

/* sel: [R][cap]; idx: [R][k] (entries past count[r] are set to -1); count: [R] */
int hco_topk(const float* sel, int64_t R, int64_t cap, const int64_t* n, int64_t k,
             int32_t* idx, int32_t* count) {
  if (k < 0) return HCO_ERR_BAD_ARG;
  int err = 0;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < R; ++r) {
    for (int64_t j = 0; j < n[r]; ++j) if (isnan(sel[r * cap + j])) err = 1;
    int c = topk_row(sel + r * cap, n[r], k, idx + r * k);
    for (int64_t j = c; j < k; ++j) idx[r * k + j] = -1;
    count[r] = c;
  }
  return err ? HCO_ERR_NAN : HCO_OK;
}

/* ------------------------------------------------------------- attend --- */

/* For every query head hq = r*G+g:
 *   l_i = z~[hq, idx_i] * sm_scale          (fp32, z~ recomputed from the codes)
 *   p_i = exp(l_i - max l), a_i = p_i / sum p    (fp64)
 *   y   = sum_i a_i * V[r][pos[idx_i]]           (fp64, cast to fp32)
 * V: [R][vrows][D] fp16.  pos: [R][cap] int32 maps a resident slot to its value row.
 * w_opt: [R*G][k] fp32 softmax weights, or NULL.
 * acc_opt: [R][cap] fp32, acc[idx_i] += sum_g max((float)a_i, 1e-30f), or NULL.
 * lse_opt: [R*G] fp32 or NULL.  Given, the weights are the paper's own (Eq. 5): a_i = exp(l_i - lse),
 * the softmax over ALL resident tokens restricted to the selected ones, not renormalised. */
int hco_attend(const uint16_t* q, const uint8_t* codes, const uint16_t* scale,
               const uint16_t* zero, int64_t R, int G, int D, int bits, int gs, int64_t cap,
               const int32_t* idx, const int32_t* count, int64_t k, const int32_t* pos,
               const uint16_t* V, int64_t vrows, float sm_scale,
               float* y, float* w_opt, float* acc_opt, const float* lse_opt) {
  if (!shape_ok(D, bits, gs) || G <= 0 || G > 16) return HCO_ERR_BAD_ARG;
  const int NG = D / gs, CB = D * bits / 8;
  int err = 0;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < R; ++r) {
    int kk = count[r];
    int32_t* qfx = (int32_t*)malloc(sizeof(int32_t) * (size_t)D);
    float* l = (float*)malloc(sizeof(float) * (size_t)(kk > 0 ? kk : 1));
    double* a = (double*)malloc(sizeof(double) * (size_t)(kk > 0 ? kk : 1));
    float* wsum = (float*)calloc((size_t)(kk > 0 ? kk : 1), sizeof(float));
    for (int g = 0; g < G; ++g) {
      int64_t hq = r * G + g;
      int32_t s;
      if (hco_query_fixed(q + hq * D, D, qfx, &s) != HCO_OK) err = 1;
      float m = -INFINITY;
      for (int i = 0; i < kk; ++i) {
        int64_t j = idx[r * k + i];
        float zt = score_one(qfx, s, codes + (r * cap + j) * CB, scale + (r * cap + j) * NG,
                             zero + (r * cap + j) * NG, D, bits, gs);
        l[i] = zt * sm_scale;
        if (l[i] > m) m = l[i];
      }
      double Z = 0.0;
      for (int i = 0; i < kk; ++i) { a[i] = exp((double)l[i] - (double)m); Z += a[i]; }
      if (lse_opt) Z = exp((double)lse_opt[hq] - (double)m);     /* denominator over all resident tokens */
      double yy[512];
      for (int c = 0; c < D; ++c) yy[c] = 0.0;
      for (int i = 0; i < kk; ++i) {
        a[i] /= Z;
        int64_t row = pos[r * cap + idx[r * k + i]];
        if (row < 0 || row >= vrows) { err = 1; continue; }
        const uint16_t* v = V + (r * vrows + row) * D;
        for (int c = 0; c < D; ++c) yy[c] += a[i] * (double)hco_h2f(v[c]);
        if (w_opt) w_opt[hq * k + i] = (float)a[i];
        float af = (float)a[i];
        if (af < 1e-30f) af = 1e-30f;
        wsum[i] += af;
      }
      for (int c = 0; c < D; ++c) y[hq * D + c] = (float)yy[c];
      if (w_opt) for (int64_t i = kk; i < k; ++i) w_opt[hq * k + i] = 0.0f;
    }
    if (acc_opt)
      for (int i = 0; i < kk; ++i) acc_opt[r * cap + idx[r * k + i]] += wsum[i];
    free(qfx); free(l); free(a); free(wsum);
  }
  return err ? HCO_ERR_BAD_ARG : HCO_OK;
}

/* -------------------------------------------------------------- evict --- */

/* Per row with n > M: slots [n-Rp, n) are kept unconditionally; from [0, n-Rp)
 * keep the M-Rp highest by (acc descending, slot ascending).  Kept slots move,
 * in ascending old-slot order, to slots 0..M-1 of codes/scale/zero/acc/pos.
 * kept: [R][M] old slots (-1 past n_new[r]).  Rows with n <= M are unchanged
 * and report kept = 0..n-1. */
int hco_evict(uint8_t* codes, uint16_t* scale, uint16_t* zero, float* acc, int32_t* pos,
              int64_t R, int D, int bits, int gs, int64_t cap, const int64_t* n,
              int64_t M, int64_t Rp, int32_t* kept, int64_t* n_new) {
  if (!shape_ok(D, bits, gs) || M < 0 || Rp < 0 || Rp > M) return HCO_ERR_BAD_ARG;
  const int NG = D / gs, CB = D * bits / 8;
  int err = 0;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < R; ++r) {
    int64_t nr = n[r];
    int32_t* kp = kept + r * M;
    if (nr <= M) {
      for (int64_t j = 0; j < M; ++j) kp[j] = j < nr ? (int32_t)j : -1;
      n_new[r] = nr;
      continue;
    }
    for (int64_t j = 0; j < nr; ++j) if (isnan(acc[r * cap + j])) err = 1;
    int64_t nfree = nr - Rp;
    int c = topk_row(acc + r * cap, nfree, M - Rp, kp);      /* ascending old slots */
    for (int64_t j = 0; j < Rp; ++j) kp[c + j] = (int32_t)(nfree + j);
    /* stable compaction: destination d <= source, ascending, so in place is safe */
    for (int64_t d = 0; d < M; ++d) {
      int64_t s = kp[d];
      if (s == d) continue;
      memmove(codes + (r * cap + d) * CB, codes + (r * cap + s) * CB, (size_t)CB);
      memmove(scale + (r * cap + d) * NG, scale + (r * cap + s) * NG, sizeof(uint16_t) * NG);
      memmove(zero + (r * cap + d) * NG, zero + (r * cap + s) * NG, sizeof(uint16_t) * NG);
      acc[r * cap + d] = acc[r * cap + s];
      pos[r * cap + d] = pos[r * cap + s];
    }
    n_new[r] = M;
  }
  return err ? HCO_ERR_NAN : HCO_OK;
}
