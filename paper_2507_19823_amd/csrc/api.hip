// C ABI of libhca: argument validation, layout, workspace sizing, dispatch.
#include <string.h>

#include "hca_internal.h"

namespace hca {

static thread_local int32_t g_last_hip = 0;

Tuning& tuning() {
  static Tuning t;
  return t;
}

int32_t hip_fail(hipError_t e) {
  g_last_hip = (int32_t)e;
  return HCA_ERR_HIP;
}

int32_t make_layout(const hca_shape* s, Layout* L) {
  if (s == nullptr) return HCA_ERR_BAD_ARG;
  if (s->batch < 1 || s->n_q_heads < 1 || s->n_kv_heads < 1 || s->capacity < 1) return HCA_ERR_BAD_ARG;
  if (s->n_q_heads % s->n_kv_heads != 0) return HCA_ERR_BAD_ARG;
  if (s->batch > kMaxBatch) return HCA_ERR_UNSUPPORTED;
  if (s->head_dim != kHeadDim) return HCA_ERR_UNSUPPORTED;
  const int gqa = s->n_q_heads / s->n_kv_heads;
  if (!(gqa == 1 || gqa == 2 || gqa == 4)) return HCA_ERR_UNSUPPORTED;
  if (!((s->bits == 4 && s->group == 32) || (s->bits == 2 && s->group == 64))) return HCA_ERR_UNSUPPORTED;
  if (s->capacity > (int64_t)1 << 30) return HCA_ERR_UNSUPPORTED;  // slots are int32
  L->bits = s->bits;
  L->group = s->group;
  L->ng = kHeadDim / s->group;
  L->tpb = kBlockBytes / (kHeadDim * s->bits / 8);
  L->batch = s->batch;
  L->n_kv_heads = s->n_kv_heads;
  L->rows = s->batch * s->n_kv_heads;
  L->gqa = gqa;
  L->cap = s->capacity;
  L->nblk = (s->capacity + L->tpb - 1) / L->tpb;
  L->meta_off = (int64_t)L->rows * L->codes_row_bytes();
  return HCA_OK;
}

int32_t load_nres(const Layout& L, const int64_t* n_resident, NRes* out, int64_t* nmax) {
  if (n_resident == nullptr) return HCA_ERR_BAD_ARG;
  int64_t mx = 0;
  for (int b = 0; b < kMaxBatch; ++b) out->n[b] = 0;
  for (int b = 0; b < L.batch; ++b) {
    if (n_resident[b] < 0) return HCA_ERR_BAD_ARG;
    if (n_resident[b] > L.cap) return HCA_ERR_CAPACITY;
    out->n[b] = n_resident[b];
    if (n_resident[b] > mx) mx = n_resident[b];
  }
  *nmax = mx;
  return HCA_OK;
}

}  // namespace hca

using namespace hca;

extern "C" {

const char* hca_version(void) { return "hca 0.1 (gfx950)"; }

int32_t hca_tune(const char* name, int32_t value) {
  if (name == nullptr) return HCA_ERR_BAD_ARG;
  Tuning& t = tuning();
  // every knob has a closed range: the kernels' buffers (wave stamps, partial sums) are sized for it
  if (!strcmp(name, "gather_wgs")) {
    if (value < 0 || value > 1024) return HCA_ERR_BAD_ARG;
    t.gather_wgs = value;
  } else if (!strcmp(name, "gather_unroll")) {
    if (value < 0 || value > 4) return HCA_ERR_BAD_ARG;
    t.gather_unroll = value;
  } else if (!strcmp(name, "score_bpw")) {
    if (value != 0 && (value < kScoreBpwMin || value > kScoreBpwMax)) return HCA_ERR_BAD_ARG;
    t.score_bpw = value;
  } else if (!strcmp(name, "score_depth")) {
    if (!(value == 0 || value == 4 || value == 8)) return HCA_ERR_BAD_ARG;
    t.score_depth = value;
  } else if (!strcmp(name, "select_wg")) {
    if (!(value == 0 || value == 256 || value == 1024)) return HCA_ERR_BAD_ARG;
    t.select_wg = value;
  } else if (!strcmp(name, "host_isa")) {
    if (!(value == 0 || value == 2)) return HCA_ERR_BAD_ARG;
    t.host_isa = value;
  } else if (!strcmp(name, "host_spin_us")) {
    t.host_spin_us = value < 0 ? 0 : value;
  } else {
    return HCA_ERR_BAD_ARG;
  }
  return HCA_OK;
}

int32_t hca_last_hip_error(void) { return g_last_hip; }

size_t hca_kcache_bytes(const hca_shape* shape) {
  Layout L;
  if (make_layout(shape, &L) != HCA_OK) return 0;
  return (size_t)L.total_bytes();
}

size_t hca_workspace_bytes(const hca_shape* shape, int64_t k_max, int64_t m_max) {
  Layout L;
  if (make_layout(shape, &L) != HCA_OK) return 0;
  if (k_max < 1) k_max = 1;
  if (m_max < 1) m_max = 1;
  if (k_max > L.cap) k_max = L.cap;
  if (m_max > L.cap) m_max = L.cap;
  size_t a = topk_workspace_bytes(L.rows, L.cap);
  size_t b = attend_workspace_bytes(L, k_max);
  size_t c = evict_workspace_bytes(L, m_max);
  size_t d = score_workspace_bytes(L);
  size_t m = a > b ? a : b;
  if (d > m) m = d;
  return (m > c ? m : c) + 256;
}

int32_t hca_quantize_keys(const hca_shape* shape, void* kcache, const void* k_new_f16, int64_t T,
                          const int64_t* n_resident, float* acc_opt, int32_t* pos_opt,
                          const int64_t* value_row0, void* stream) {
  Layout L;
  int32_t rc = make_layout(shape, &L);
  if (rc != HCA_OK) return rc;
  if (kcache == nullptr || T < 0 || (T > 0 && k_new_f16 == nullptr)) return HCA_ERR_BAD_ARG;
  NRes nr;
  int64_t nmax;
  rc = load_nres(L, n_resident, &nr, &nmax);
  if (rc != HCA_OK) return rc;
  for (int b = 0; b < L.batch; ++b)
    if (nr.n[b] + T > L.cap) return HCA_ERR_CAPACITY;
  NRes vrow0;
  for (int b = 0; b < kMaxBatch; ++b) vrow0.n[b] = 0;
  if (pos_opt != nullptr) {
    if (value_row0 == nullptr) return HCA_ERR_BAD_ARG;
    for (int b = 0; b < L.batch; ++b) {
      if (value_row0[b] < 0 || value_row0[b] + T > (int64_t)INT32_MAX) return HCA_ERR_BAD_ARG;
      vrow0.n[b] = value_row0[b];
    }
  }
  return launch_quantize(L, kcache, k_new_f16, T, nr, acc_opt, pos_opt, vrow0, (hipStream_t)stream);
}

int32_t hca_score_qkeys(const hca_shape* shape, const void* kcache, const void* q_f16,
                        const int64_t* n_resident, float* sel, float* z_opt, void* workspace, void* stream) {
  (void)workspace;
  Layout L;
  int32_t rc = make_layout(shape, &L);
  if (rc != HCA_OK) return rc;
  if (kcache == nullptr || q_f16 == nullptr || sel == nullptr) return HCA_ERR_BAD_ARG;
  NRes nr;
  int64_t nmax;
  rc = load_nres(L, n_resident, &nr, &nmax);
  if (rc != HCA_OK) return rc;
  return launch_score(L, kcache, q_f16, nr, nmax, sel, z_opt, (hipStream_t)stream);
}

int32_t hca_topk(const hca_shape* shape, const float* sel, const int64_t* n_resident, int32_t k,
                 int32_t* idx, int32_t* count, void* workspace, void* stream) {
  Layout L;
  int32_t rc = make_layout(shape, &L);
  if (rc != HCA_OK) return rc;
  if (sel == nullptr || idx == nullptr || count == nullptr || workspace == nullptr) return HCA_ERR_BAD_ARG;
  if (k < 1 || k > L.cap) return HCA_ERR_CAPACITY;
  NRes nr;
  int64_t nmax;
  rc = load_nres(L, n_resident, &nr, &nmax);
  if (rc != HCA_OK) return rc;
  return launch_topk(L, sel, nr, nmax, k, idx, count, workspace, (hipStream_t)stream);
}

int32_t hca_score_topk(const hca_shape* shape, const void* kcache, const void* q_f16, const int64_t* n_resident,
                       int32_t k, int32_t* idx, int32_t* count, void* workspace, void* stream) {
  Layout L;
  int32_t rc = make_layout(shape, &L);
  if (rc != HCA_OK) return rc;
  if (kcache == nullptr || q_f16 == nullptr || idx == nullptr || count == nullptr || workspace == nullptr)
    return HCA_ERR_BAD_ARG;
  if (k < 1 || k > L.cap) return HCA_ERR_CAPACITY;
  NRes nr;
  int64_t nmax;
  rc = load_nres(L, n_resident, &nr, &nmax);
  if (rc != HCA_OK) return rc;
  return launch_score_topk(L, kcache, q_f16, nr, nmax, k, idx, count, workspace, (hipStream_t)stream);
}

int32_t hca_score_topk_report(const hca_shape* shape, const int64_t* n_resident, void* workspace, int32_t* candidates,
                              int32_t* rescanned, void* stream) {
  Layout L;
  int32_t rc = make_layout(shape, &L);
  if (rc != HCA_OK) return rc;
  if (workspace == nullptr || candidates == nullptr || rescanned == nullptr) return HCA_ERR_BAD_ARG;
  NRes nr;
  int64_t nmax;
  rc = load_nres(L, n_resident, &nr, &nmax);
  if (rc != HCA_OK) return rc;
  return launch_select_report(L, nr, nmax, workspace, candidates, rescanned, (hipStream_t)stream);
}

int32_t hca_score_topk_monitor(const hca_shape* shape, void* workspace, int32_t* out, int32_t reset, void* stream) {
  Layout L;
  const int32_t rc = make_layout(shape, &L);
  if (rc != HCA_OK) return rc;
  if (workspace == nullptr) return HCA_ERR_BAD_ARG;
  return launch_select_monitor(L, workspace, out, reset != 0, (hipStream_t)stream);
}

int32_t hca_score_qkeys_lse(const hca_shape* shape, const void* kcache, const void* q_f16,
                            const int64_t* n_resident, float sm_scale, float* sel, float* lse, void* workspace,
                            void* stream) {
  Layout L;
  int32_t rc = make_layout(shape, &L);
  if (rc != HCA_OK) return rc;
  if (kcache == nullptr || q_f16 == nullptr || sel == nullptr || lse == nullptr || workspace == nullptr)
    return HCA_ERR_BAD_ARG;
  if (!(sm_scale > 0.0f)) return HCA_ERR_BAD_ARG;
  NRes nr;
  int64_t nmax;
  rc = load_nres(L, n_resident, &nr, &nmax);
  if (rc != HCA_OK) return rc;
  return launch_score_lse(L, kcache, q_f16, nr, nmax, sm_scale, sel, lse, workspace, (hipStream_t)stream);
}

int32_t hca_attend_gathered_global(const hca_shape* shape, const void* kcache, const void* q_f16, const int32_t* idx,
                                   const int32_t* count, int32_t k, float sm_scale, const float* lse, float* y,
                                   float* acc_opt, void* workspace, void* stream) {
  Layout L;
  int32_t rc = make_layout(shape, &L);
  if (rc != HCA_OK) return rc;
  if (kcache == nullptr || q_f16 == nullptr || idx == nullptr || count == nullptr || lse == nullptr || y == nullptr ||
      workspace == nullptr)
    return HCA_ERR_BAD_ARG;
  if (k < 1 || k > L.cap || k > 64 * 256) return HCA_ERR_CAPACITY;
  return launch_attend_gathered(L, kcache, q_f16, idx, count, k, sm_scale, y, acc_opt, workspace, (hipStream_t)stream,
                                lse);
}

int32_t hca_attend_weights(const hca_shape* shape, const void* kcache, const void* q_f16, const int32_t* idx,
                           const int32_t* count, int32_t k, const int32_t* pos, float sm_scale, const float* lse_opt,
                           void* w_f16, int32_t* vrow, float* acc_opt, void* workspace, void* stream) {
  Layout L;
  int32_t rc = make_layout(shape, &L);
  if (rc != HCA_OK) return rc;
  if (kcache == nullptr || q_f16 == nullptr || idx == nullptr || count == nullptr || pos == nullptr ||
      w_f16 == nullptr || vrow == nullptr || workspace == nullptr)
    return HCA_ERR_BAD_ARG;
  if (k < 1 || k > L.cap || k > 64 * 256) return HCA_ERR_CAPACITY;
  return launch_attend_weights(L, kcache, q_f16, idx, count, k, pos, sm_scale, lse_opt, w_f16, vrow, acc_opt, workspace,
                               (hipStream_t)stream);
}

int32_t hca_topp(const hca_shape* shape, const float* sel, const int64_t* n_resident, float sm_scale, double tau,
                 int32_t k_max, int32_t* idx, int32_t* count, uint64_t* mass_opt, void* workspace, void* stream) {
  Layout L;
  int32_t rc = make_layout(shape, &L);
  if (rc != HCA_OK) return rc;
  if (sel == nullptr || idx == nullptr || count == nullptr || workspace == nullptr) return HCA_ERR_BAD_ARG;
  if (!(tau > 0.0) || !(sm_scale > 0.0f)) return HCA_ERR_BAD_ARG;
  if (k_max < 1 || k_max > L.cap) return HCA_ERR_CAPACITY;
  NRes nr;
  int64_t nmax;
  rc = load_nres(L, n_resident, &nr, &nmax);
  if (rc != HCA_OK) return rc;
  return launch_topp(L, sel, nr, nmax, sm_scale, tau, k_max, idx, count, mass_opt, workspace, (hipStream_t)stream);
}

int32_t hca_sparse_attend(const hca_shape* shape, const void* kcache, const void* q_f16, const int32_t* idx,
                          const int32_t* count, int32_t k, const int32_t* pos, const void* v_host,
                          int64_t host_stride, int64_t n_host_rows, const void* v_hbm, int64_t hbm_stride,
                          float sm_scale, float* y, float* acc_opt, void* workspace, void* gather_stream,
                          void* stream) {
  Layout L;
  int32_t rc = make_layout(shape, &L);
  if (rc != HCA_OK) return rc;
  if (kcache == nullptr || q_f16 == nullptr || idx == nullptr || count == nullptr || pos == nullptr ||
      y == nullptr || workspace == nullptr)
    return HCA_ERR_BAD_ARG;
  if (k < 1 || k > L.cap || k > 64 * 256) return HCA_ERR_CAPACITY;
  if (n_host_rows < 0 || host_stride < 0 || hbm_stride < 0) return HCA_ERR_BAD_ARG;
  if (n_host_rows > 0 && (v_host == nullptr || host_stride < n_host_rows)) return HCA_ERR_BAD_ARG;
  if (v_host == nullptr && v_hbm == nullptr) return HCA_ERR_BAD_ARG;
  return launch_attend(L, kcache, q_f16, idx, count, k, pos, v_host, host_stride, n_host_rows, v_hbm,
                       hbm_stride, sm_scale, y, acc_opt, workspace, (hipStream_t)gather_stream,
                       (hipStream_t)stream);
}

int32_t hca_gather_values(const hca_shape* shape, const int32_t* idx, const int32_t* count, int32_t k,
                          const int32_t* pos, const void* v_host, int64_t host_stride, int64_t n_host_rows,
                          const void* v_hbm, int64_t hbm_stride, void* workspace, void* stream) {
  Layout L;
  int32_t rc = make_layout(shape, &L);
  if (rc != HCA_OK) return rc;
  if (idx == nullptr || count == nullptr || pos == nullptr || workspace == nullptr) return HCA_ERR_BAD_ARG;
  if (k < 1 || k > L.cap || k > 64 * 256) return HCA_ERR_CAPACITY;
  if (n_host_rows < 0 || host_stride < 0 || hbm_stride < 0) return HCA_ERR_BAD_ARG;
  if (n_host_rows > 0 && (v_host == nullptr || host_stride < n_host_rows)) return HCA_ERR_BAD_ARG;
  if (v_host == nullptr && v_hbm == nullptr) return HCA_ERR_BAD_ARG;
  return launch_gather(L, idx, count, k, pos, v_host, host_stride, n_host_rows, v_hbm, hbm_stride, workspace,
                       (hipStream_t)stream);
}

int32_t hca_attend_gathered(const hca_shape* shape, const void* kcache, const void* q_f16, const int32_t* idx,
                            const int32_t* count, int32_t k, float sm_scale, float* y, float* acc_opt,
                            void* workspace, void* stream) {
  Layout L;
  int32_t rc = make_layout(shape, &L);
  if (rc != HCA_OK) return rc;
  if (kcache == nullptr || q_f16 == nullptr || idx == nullptr || count == nullptr || y == nullptr ||
      workspace == nullptr)
    return HCA_ERR_BAD_ARG;
  if (k < 1 || k > L.cap || k > 64 * 256) return HCA_ERR_CAPACITY;
  return launch_attend_gathered(L, kcache, q_f16, idx, count, k, sm_scale, y, acc_opt, workspace,
                                (hipStream_t)stream);
}

int32_t hca_evict(const hca_shape* shape, void* kcache, float* acc, int32_t* pos, const int64_t* n_resident,
                  int64_t M, int64_t n_protect, int32_t* kept_opt, void* workspace, void* kcache_dst,
                  float* acc_dst, int32_t* pos_dst, void* stream) {
  Layout L;
  int32_t rc = make_layout(shape, &L);
  if (rc != HCA_OK) return rc;
  if (kcache == nullptr || acc == nullptr || pos == nullptr || workspace == nullptr) return HCA_ERR_BAD_ARG;
  if (M < 1 || M > L.cap || n_protect < 0 || n_protect > M) return HCA_ERR_CAPACITY;
  if (kcache_dst != nullptr && (acc_dst == nullptr || pos_dst == nullptr || kcache_dst == kcache ||
                                acc_dst == acc || pos_dst == pos))
    return HCA_ERR_BAD_ARG;
  if (kcache_dst == nullptr && (acc_dst != nullptr || pos_dst != nullptr)) return HCA_ERR_BAD_ARG;
  NRes nr;
  int64_t nmax;
  rc = load_nres(L, n_resident, &nr, &nmax);
  if (rc != HCA_OK) return rc;
  return launch_evict(L, kcache, acc, pos, nr, nmax, M, n_protect, kept_opt, workspace, kcache_dst, acc_dst,
                      pos_dst, (hipStream_t)stream);
}

int32_t hca_export_kcache(const hca_shape* shape, const void* kcache, const int64_t* n_resident,
                          uint8_t* codes, void* scale_f16, void* zero_f16, void* stream) {
  Layout L;
  int32_t rc = make_layout(shape, &L);
  if (rc != HCA_OK) return rc;
  if (kcache == nullptr || codes == nullptr || scale_f16 == nullptr || zero_f16 == nullptr) return HCA_ERR_BAD_ARG;
  NRes nr;
  int64_t nmax;
  rc = load_nres(L, n_resident, &nr, &nmax);
  if (rc != HCA_OK) return rc;
  return launch_export(L, kcache, nr, codes, scale_f16, zero_f16, (hipStream_t)stream);
}

}  // extern "C"
