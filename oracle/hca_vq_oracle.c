/*
 * hca_vq_oracle.c: slow, plain CPU reference for the codebook form of the key
 * path (grouped vector quantisation, Sec. 3.1, and the table-lookup scores of
 * Sec. 3.2, Eq. 3).
 *
 * TEST INFRASTRUCTURE ONLY, like hca_oracle.c next to it: the parity oracle of
 * the hca_vq_* entry points.  Nothing in the product path links, loads or calls
 * it and it shares no code with the HIP library.  It is linked into the same
 * shared object as hca_oracle.c and uses that file's fp16 conversion.
 *
 *   hco_vq_train     codebook C in R^{g x c x dbar}: the key space is cut into g
 *                    groups of dbar = d/g channels and each group's sub-vectors
 *                    of a validation set are clustered (Lloyd's k-means), Sec. 3.1
 *   hco_vq_assign    index matrix P in Z^{n x g}: every sub-vector is replaced by
 *                    the index of its nearest centroid, Sec. 3.2 (GPU part)
 *   hco_vq_dequant   the centroids the indices stand for, Q(K)
 *   hco_vq_lut       the table T = qbar . C in R^{g x c}, Sec. 3.2
 *   hco_vq_score     z~_j = sum_i T[i, P[j, i]], Eq. 3, plus the per-KV-head
 *                    selection score (max over the query heads of the group)
 *   hco_vq_attend    softmax over the selected set and the weighted value sum of
 *                    Eq. 5 with the logits of Eq. 3; accumulated-score update
 *   hco_vq_evict     keep-M by accumulated score with stable compaction of the
 *                    index rows (the policy of hco_evict in hca_oracle.c)
 *
 * Indices are 0-based.  Everything that feeds an integer decision is single
 * fp32 operations in one fixed order, or exact integer arithmetic (compile with
 * -ffp-contract=off, no fast-math):
 *   distance   d = 0; for each channel of the group, ascending: t = x - c;
 *              d = fmaf(t, t, d).  Nearest = smallest d, ties to the lowest index.
 *   table      T = 0; for each channel ascending: T = fmaf(q, c, T).
 *   score      Eq. 3 is a sum of g table entries; the paper fixes neither its
 *              precision nor its order.  Here the sum itself is exact: the table of
 *              a query head is first put on one power-of-two grid,
 *                s = 23 - floor(log2(max |T|))   (0 for an all-zero table),
 *                Tfx = (int) rintf(ldexpf(T, s))  so that |Tfx| <= 2^24,
 *              (24 bits for the largest entry, as many as fp32 keeps), then
 *                z = ldexpf((float)(sum_i Tfx[i, P_i]), -s)
 *              with the integer sum exact, hence the same in any order.
 * Centroid means, inertia, softmax and the weighted sum accumulate in fp64.
 *
 * Parity status.  Assignment, table and scores are pinned against brute force
 * and against the identity z~ = q . Q(K)^T; the trainer against planted clusters
 * and the monotone decrease of the k-means objective.  The paper does not say
 * how centroids are initialised, how many iterations run or what happens to an
 * empty cluster: here the caller passes the seeding vectors, the iteration count
 * is an argument and an empty cluster keeps its centroid ("parity unpinned" by
 * the paper for those three choices).
 *
 * Layouts (R = batch * kv_heads rows; row r uses the codebook of KV head
 * r % n_kv; query head r*G + h belongs to row r):
 *   C  [n_kv][g][c][dbar] fp32      P  [R][cap][g] uint16
 *   T  [R*G][g][c] fp32
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define HCO_OK 0
#define HCO_ERR_BAD_ARG (-1)
#define HCO_ERR_NAN (-2)

float hco_h2f(uint16_t h);   /* hca_oracle.c */

static int vq_shape_ok(int D, int g, int c) {
  if (D <= 0 || D > 512 || g <= 0 || D % g != 0) return 0;
  if (c < 1 || c > 65536) return 0;
  return 1;
}

/* squared distance of sub-vector x[dbar] to centroid cv[dbar], fp32, channels ascending */
static float dist2(const float* x, const float* cv, int dbar) {
  float d = 0.0f;
  for (int t = 0; t < dbar; ++t) {
    float e = x[t] - cv[t];
    d = fmaf(e, e, d);
  }
  return d;
}

/* index of the nearest of c centroids (ties: lowest index); *dmin gets its distance */
static int nearest(const float* x, const float* cb, int c, int dbar, float* dmin) {
  int best = 0;
  float bd = dist2(x, cb, dbar);
  for (int cc = 1; cc < c; ++cc) {
    float d = dist2(x, cb + (size_t)cc * dbar, dbar);
    if (d < bd) { bd = d; best = cc; }
  }
  if (dmin) *dmin = bd;
  return best;
}

/* --------------------------------------------------------------- train --- */

/* Lloyd's k-means per group on the sub-vectors of kval [nval][D] (fp16 bits).
 * shared == 0: group i clusters its own nval sub-vectors; init [g][c] holds, per
 *   group, the validation tokens whose sub-vectors seed the centroids.
 * shared != 0: one codebook is trained on all g*nval sub-vectors pooled (pool
 *   entry t*g + i is sub-vector i of token t), init [c] indexes the pool, and the
 *   result is written to every group.
 * Each of `iters` rounds assigns every sub-vector to its nearest centroid and
 * moves each centroid to the mean of its members (fp64 sum in pool order, one
 * cast to fp32); a centroid without members stays.  inertia [iters + 1] (may be
 * NULL): the k-means objective (sum of squared distances, fp64 sum of the fp32
 * distances, summed over groups) at the assignment of each round and once more
 * after the last update.  C out: [g][c][dbar]. */
int hco_vq_train(const uint16_t* kval, int64_t nval, int D, int g, int c, const int32_t* init,
                 int iters, int shared, float* C, double* inertia) {
  if (!vq_shape_ok(D, g, c) || nval < 1 || iters < 0) return HCO_ERR_BAD_ARG;
  const int dbar = D / g;
  const int ncb = shared ? 1 : g;                    /* codebooks to train */
  const int64_t npool = shared ? nval * g : nval;    /* sub-vectors per codebook */
  for (int it = 0; inertia && it <= iters; ++it) inertia[it] = 0.0;
  int err = 0;
  double* iner = (double*)calloc((size_t)ncb * (size_t)(iters + 1), sizeof(double));
#pragma omp parallel for schedule(dynamic)
  for (int b = 0; b < ncb; ++b) {
    /* the pool of this codebook, fp32 */
    float* x = (float*)malloc(sizeof(float) * (size_t)npool * dbar);
    for (int64_t p = 0; p < npool; ++p) {
      int64_t t = shared ? p / g : p;
      int i = shared ? (int)(p % g) : b;
      for (int dd = 0; dd < dbar; ++dd) x[p * dbar + dd] = hco_h2f(kval[t * D + i * dbar + dd]);
    }
    float* cb = C + (size_t)b * c * dbar;
    for (int cc = 0; cc < c; ++cc) {
      int64_t s = init[(size_t)b * c + cc];
      if (s < 0 || s >= npool) { err = 1; s = 0; }
      memcpy(cb + (size_t)cc * dbar, x + s * dbar, sizeof(float) * dbar);
    }
    double* sum = (double*)malloc(sizeof(double) * (size_t)c * dbar);
    int64_t* cnt = (int64_t*)malloc(sizeof(int64_t) * (size_t)c);
    for (int it = 0; it <= iters; ++it) {
      memset(sum, 0, sizeof(double) * (size_t)c * dbar);
      memset(cnt, 0, sizeof(int64_t) * (size_t)c);
      double obj = 0.0;
      for (int64_t p = 0; p < npool; ++p) {
        float dm;
        int a = nearest(x + p * dbar, cb, c, dbar, &dm);
        obj += (double)dm;
        cnt[a] += 1;
        for (int dd = 0; dd < dbar; ++dd) sum[(size_t)a * dbar + dd] += (double)x[p * dbar + dd];
      }
      iner[(size_t)b * (iters + 1) + it] = obj;
      if (it == iters) break;                        /* last pass only measures */
      for (int cc = 0; cc < c; ++cc)
        if (cnt[cc] > 0)
          for (int dd = 0; dd < dbar; ++dd)
            cb[(size_t)cc * dbar + dd] = (float)(sum[(size_t)cc * dbar + dd] / (double)cnt[cc]);
    }
    free(x); free(sum); free(cnt);
  }
  if (shared)
    for (int i = 1; i < g; ++i) memcpy(C + (size_t)i * c * dbar, C, sizeof(float) * (size_t)c * dbar);
  for (int b = 0; inertia && b < ncb; ++b)
    for (int it = 0; it <= iters; ++it) inertia[it] += iner[(size_t)b * (iters + 1) + it];
  free(iner);
  return err ? HCO_ERR_BAD_ARG : HCO_OK;
}

/* -------------------------------------------------------------- assign --- */

/* Appends T tokens per row: P[r][n[r] + t][i] = nearest centroid of sub-vector i of
 * k_new[r][t] in codebook C[r % n_kv][i].  n is updated. */
int hco_vq_assign(const uint16_t* k_new, int64_t R, int64_t T, int D, int g, int c, int n_kv,
                  const float* C, int64_t cap, int64_t* n, uint16_t* P) {
  if (!vq_shape_ok(D, g, c) || R < 0 || T < 0 || n_kv < 1) return HCO_ERR_BAD_ARG;
  const int dbar = D / g;
  for (int64_t r = 0; r < R; ++r) if (n[r] < 0 || n[r] + T > cap) return HCO_ERR_BAD_ARG;
  int err = 0;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < R; ++r) {
    const float* cbr = C + (size_t)(r % n_kv) * g * c * dbar;
    float x[512];
    for (int64_t t = 0; t < T; ++t) {
      const uint16_t* src = k_new + (r * T + t) * D;
      for (int ch = 0; ch < D; ++ch) {
        x[ch] = hco_h2f(src[ch]);
        if (isnan(x[ch])) err = 1;
      }
      uint16_t* dst = P + (r * cap + n[r] + t) * g;
      for (int i = 0; i < g; ++i)
        dst[i] = (uint16_t)nearest(x + i * dbar, cbr + (size_t)i * c * dbar, c, dbar, NULL);
    }
  }
  for (int64_t r = 0; r < R; ++r) n[r] += T;
  return err ? HCO_ERR_NAN : HCO_OK;
}

/* Q(K): out[r][j][D] fp32 = the centroids the indices of slot j stand for. */
int hco_vq_dequant(const uint16_t* P, int64_t R, int D, int g, int c, int n_kv, const float* C,
                   int64_t cap, const int64_t* n, float* out) {
  if (!vq_shape_ok(D, g, c) || n_kv < 1) return HCO_ERR_BAD_ARG;
  const int dbar = D / g;
  for (int64_t r = 0; r < R; ++r) {
    const float* cbr = C + (size_t)(r % n_kv) * g * c * dbar;
    for (int64_t j = 0; j < n[r]; ++j)
      for (int i = 0; i < g; ++i) {
        int a = P[(r * cap + j) * g + i];
        if (a >= c) return HCO_ERR_BAD_ARG;
        memcpy(out + (r * cap + j) * D + i * dbar, cbr + ((size_t)i * c + a) * dbar, sizeof(float) * dbar);
      }
  }
  return HCO_OK;
}

/* ----------------------------------------------------------------- lut --- */

/* T[hq][i][cc] = qbar_i . C[i][cc] for every query head hq = r*G + h. */
int hco_vq_lut(const uint16_t* q, int64_t R, int G, int D, int g, int c, int n_kv, const float* C,
               float* T) {
  if (!vq_shape_ok(D, g, c) || G < 1 || G > 16 || n_kv < 1) return HCO_ERR_BAD_ARG;
  const int dbar = D / g;
  for (int64_t hq = 0; hq < R * G; ++hq) {
    const float* cbr = C + (size_t)((hq / G) % n_kv) * g * c * dbar;
    for (int i = 0; i < g; ++i)
      for (int cc = 0; cc < c; ++cc) {
        float t = 0.0f;
        for (int dd = 0; dd < dbar; ++dd)
          t = fmaf(hco_h2f(q[hq * D + i * dbar + dd]), cbr[((size_t)i * c + cc) * dbar + dd], t);
        T[(hq * g + i) * c + cc] = t;
      }
  }
  return HCO_OK;
}

/* --------------------------------------------------------------- score --- */

/* Fixed-point image of the tables of nq query heads: T [nq][g][c] -> Tfx, sexp [nq].
 * Returns HCO_ERR_NAN when a table holds a NaN or an infinity. */
int hco_vq_lut_fx(const float* T, int64_t nq, int g, int c, int32_t* Tfx, int32_t* sexp) {
  if (g < 1 || c < 1) return HCO_ERR_BAD_ARG;
  const size_t per = (size_t)g * c;
  for (int64_t hq = 0; hq < nq; ++hq) {
    const float* t = T + (size_t)hq * per;
    float amax = 0.0f;
    for (size_t e = 0; e < per; ++e) {
      if (isnan(t[e]) || isinf(t[e])) return HCO_ERR_NAN;
      if (fabsf(t[e]) > amax) amax = fabsf(t[e]);
    }
    const int s = amax == 0.0f ? 0 : 23 - ilogbf(amax);
    sexp[hq] = s;
    for (size_t e = 0; e < per; ++e) Tfx[(size_t)hq * per + e] = (int32_t)rintf(ldexpf(t[e], s));
  }
  return HCO_OK;
}

static float vq_score_one(const int32_t* Tfx_hq, int s, const uint16_t* prow, int g, int c) {
  int64_t sum = 0;
  for (int i = 0; i < g; ++i) sum += Tfx_hq[(size_t)i * c + prow[i]];
  return ldexpf((float)sum, -s);
}

/* sel [R][cap] (entries >= n[r] untouched), z_opt [R*G][cap] or NULL. */
int hco_vq_score(const float* T, const uint16_t* P, int64_t R, int G, int g, int c, int64_t cap,
                 const int64_t* n, float* sel, float* z_opt) {
  if (g < 1 || c < 1 || G < 1 || G > 16) return HCO_ERR_BAD_ARG;
  int32_t* Tfx = (int32_t*)malloc(sizeof(int32_t) * (size_t)R * G * g * c);
  int32_t* sexp = (int32_t*)malloc(sizeof(int32_t) * (size_t)R * G);
  int rc = hco_vq_lut_fx(T, R * G, g, c, Tfx, sexp);
  if (rc != HCO_OK) { free(Tfx); free(sexp); return rc; }
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < R; ++r) {
    for (int64_t j = 0; j < n[r]; ++j) {
      const uint16_t* prow = P + (r * cap + j) * g;
      float best = -INFINITY;
      for (int h = 0; h < G; ++h) {
        float z = vq_score_one(Tfx + (size_t)(r * G + h) * g * c, sexp[r * G + h], prow, g, c);
        if (z_opt) z_opt[(r * G + h) * cap + j] = z;
        if (z > best) best = z;
      }
      sel[r * cap + j] = best;
    }
  }
  free(Tfx); free(sexp);
  return HCO_OK;
}

/* -------------------------------------------------------------- attend --- */

/* As hco_attend of hca_oracle.c with the logits of Eq. 3:
 *   l_i = z~[hq, idx_i] * sm_scale, p_i = exp(l_i - max l), a_i = p_i / sum p (fp64),
 *   y = sum_i a_i * V[r][pos[idx_i]] (fp64, cast to fp32),
 *   acc[idx_i] += sum_h max((float)a_i, 1e-30f). */
int hco_vq_attend(const float* T, const uint16_t* P, int64_t R, int G, int D, int g, int c,
                  int64_t cap, const int32_t* idx, const int32_t* count, int64_t k,
                  const int32_t* pos, const uint16_t* V, int64_t vrows, float sm_scale, float* y,
                  float* w_opt, float* acc_opt) {
  if (!vq_shape_ok(D, g, c) || G < 1 || G > 16) return HCO_ERR_BAD_ARG;
  int32_t* Tfx = (int32_t*)malloc(sizeof(int32_t) * (size_t)R * G * g * c);
  int32_t* sexp = (int32_t*)malloc(sizeof(int32_t) * (size_t)R * G);
  int rc = hco_vq_lut_fx(T, R * G, g, c, Tfx, sexp);
  if (rc != HCO_OK) { free(Tfx); free(sexp); return rc; }
  int err = 0;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < R; ++r) {
    int kk = count[r];
    float* l = (float*)malloc(sizeof(float) * (size_t)(kk > 0 ? kk : 1));
    double* a = (double*)malloc(sizeof(double) * (size_t)(kk > 0 ? kk : 1));
    float* wsum = (float*)calloc((size_t)(kk > 0 ? kk : 1), sizeof(float));
    for (int h = 0; h < G; ++h) {
      int64_t hq = r * G + h;
      float m = -INFINITY;
      for (int i = 0; i < kk; ++i) {
        int64_t j = idx[r * k + i];
        l[i] = vq_score_one(Tfx + (size_t)hq * g * c, sexp[hq], P + (r * cap + j) * g, g, c) * sm_scale;
        if (l[i] > m) m = l[i];
      }
      double Z = 0.0;
      for (int i = 0; i < kk; ++i) { a[i] = exp((double)l[i] - (double)m); Z += a[i]; }
      double yy[512];
      for (int ch = 0; ch < D; ++ch) yy[ch] = 0.0;
      for (int i = 0; i < kk; ++i) {
        a[i] /= Z;
        int64_t row = pos[r * cap + idx[r * k + i]];
        if (row < 0 || row >= vrows) { err = 1; continue; }
        const uint16_t* v = V + (r * vrows + row) * D;
        for (int ch = 0; ch < D; ++ch) yy[ch] += a[i] * (double)hco_h2f(v[ch]);
        if (w_opt) w_opt[hq * k + i] = (float)a[i];
        float af = (float)a[i];
        if (af < 1e-30f) af = 1e-30f;
        wsum[i] += af;
      }
      for (int ch = 0; ch < D; ++ch) y[hq * D + ch] = (float)yy[ch];
      if (w_opt) for (int64_t i = kk; i < k; ++i) w_opt[hq * k + i] = 0.0f;
    }
    if (acc_opt)
      for (int i = 0; i < kk; ++i) acc_opt[r * cap + idx[r * k + i]] += wsum[i];
    free(l); free(a); free(wsum);
  }
  free(Tfx); free(sexp);
  return err ? HCO_ERR_BAD_ARG : HCO_OK;
}

/* --------------------------------------------------------------- evict --- */

int hco_topk(const float* sel, int64_t R, int64_t cap, const int64_t* n, int64_t k, int32_t* idx,
             int32_t* count);   /* hca_oracle.c */

/* Accumulated-score eviction of a codebook cache: the keep-set and the order are those of
 * hco_evict in hca_oracle.c (newest Rp slots kept; of the others the M - Rp highest acc, ties to
 * the lower slot; kept slots move in ascending old-slot order to slots 0..M-1); the rows that
 * move are index rows.  kept: [R][M] old slots (-1 past n_new[r]); rows with n <= M unchanged. */
int hco_vq_evict(uint16_t* P, float* acc, int32_t* pos, int64_t R, int g, int64_t cap,
                 const int64_t* n, int64_t M, int64_t Rp, int32_t* kept, int64_t* n_new) {
  if (g < 1 || M < 0 || Rp < 0 || Rp > M) return HCO_ERR_BAD_ARG;
  int err = 0;
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
    int32_t c = 0;
    if (M - Rp > 0 && hco_topk(acc + r * cap, 1, cap, &nfree, M - Rp, kp, &c) != HCO_OK) err = 1;
    for (int64_t j = 0; j < Rp; ++j) kp[c + j] = (int32_t)(nfree + j);
    for (int64_t d = 0; d < M; ++d) {           /* destination <= source, ascending: in place is safe */
      int64_t s = kp[d];
      if (s == d) continue;
      memmove(P + (r * cap + d) * g, P + (r * cap + s) * g, sizeof(uint16_t) * (size_t)g);
      acc[r * cap + d] = acc[r * cap + s];
      pos[r * cap + d] = pos[r * cap + s];
    }
    n_new[r] = M;
  }
  return err ? HCO_ERR_NAN : HCO_OK;
}
