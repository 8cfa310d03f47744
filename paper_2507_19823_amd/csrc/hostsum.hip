// The host half of the paper's CPU-GPU split (Sec. 3.2 "CPU part", Eq. 5): the GPU hands over, per selected
// token, its value-row number and one 2-byte weight per query head (hca_attend_weights); the host forms
// y = sum_i w_i V_i from the value store that never leaves host memory.  Host code only.
#include <cstring>
#include <thread>
#include <vector>

#include "hca_internal.h"

namespace hca {

static inline float half_to_float(uint16_t h) {
  _Float16 v;
  std::memcpy(&v, &h, 2);
  return (float)v;
}

// y_part[G][128] += sum over selected tokens [i0, i1) of one row
static void sum_range(int G, int32_t k, const int32_t* vrow, const uint16_t* w /*[G][k]*/, const uint16_t* v_row0,
                      int64_t i0, int64_t i1, float* y_part) {
  for (int64_t i = i0; i < i1; ++i) {
    const int32_t r = vrow[i];
    if (r < 0) continue;
    const _Float16* v = reinterpret_cast<const _Float16*>(v_row0) + (int64_t)r * kHeadDim;
    if (i + 4 < i1 && vrow[i + 4] >= 0)            // the rows are scattered: ask for one ahead
      __builtin_prefetch(v_row0 + (int64_t)vrow[i + 4] * kHeadDim);
    float vf[kHeadDim];
    for (int c = 0; c < kHeadDim; ++c) vf[c] = (float)v[c];
    for (int h = 0; h < G; ++h) {
      const float wh = half_to_float(w[(int64_t)h * k + i]);
      float* __restrict__ y = y_part + h * kHeadDim;
      for (int c = 0; c < kHeadDim; ++c) y[c] += wh * vf[c];
    }
  }
}

}  // namespace hca

using namespace hca;

extern "C" int32_t hca_host_weighted_sum(const hca_shape* shape, const int32_t* vrow, const int32_t* count, int32_t k,
                                         const void* w_f16, const void* v_host, int64_t host_stride, float* y,
                                         int32_t n_threads) {
  Layout L;
  hca_shape s;
  if (shape == nullptr) return HCA_ERR_BAD_ARG;
  s = *shape;
  s.bits = 4;
  s.group = 32;                                   // the code format plays no part on the host side
  int32_t rc = make_layout(&s, &L);
  if (rc != HCA_OK) return rc;
  if (vrow == nullptr || count == nullptr || w_f16 == nullptr || v_host == nullptr || y == nullptr) return HCA_ERR_BAD_ARG;
  if (k < 1 || host_stride < 1) return HCA_ERR_BAD_ARG;
  if (n_threads < 1) n_threads = 1;
  if (n_threads > 64) n_threads = 64;
  const int G = L.gqa;
  // tasks: every row cut into `parts` ranges of its selected tokens, partial sums added up afterwards
  int parts = (n_threads + L.rows - 1) / L.rows;
  if (parts < 1) parts = 1;
  const int ntask = L.rows * parts;
  std::vector<float> partial((size_t)ntask * G * kHeadDim, 0.0f);
  auto work = [&](int t0) {
    for (int t = t0; t < ntask; t += n_threads) {
      const int row = t / parts, part = t % parts;
      int64_t cnt = count[row];
      if (cnt > k) cnt = k;
      const int64_t per = (cnt + parts - 1) / parts;
      int64_t i0 = per * part, i1 = i0 + per;
      if (i1 > cnt) i1 = cnt;
      if (i0 < i1)
        sum_range(G, k, vrow + (int64_t)row * k, (const uint16_t*)w_f16 + (int64_t)row * G * k,
                  (const uint16_t*)v_host + (int64_t)row * host_stride * kHeadDim, i0, i1,
                  &partial[(size_t)t * G * kHeadDim]);
    }
  };
  for (int row = 0; row < L.rows; ++row) {
    int64_t cnt = count[row] < k ? count[row] : k;
    for (int64_t i = 0; i < cnt; ++i)
      if (vrow[(int64_t)row * k + i] >= host_stride) return HCA_ERR_CAPACITY;
  }
  std::vector<std::thread> pool;
  for (int t = 1; t < n_threads; ++t) pool.emplace_back(work, t);
  work(0);
  for (auto& th : pool) th.join();
  for (int row = 0; row < L.rows; ++row)
    for (int e = 0; e < G * kHeadDim; ++e) {
      float acc = 0.0f;
      for (int part = 0; part < parts; ++part) acc += partial[((size_t)row * parts + part) * G * kHeadDim + e];
      y[(int64_t)row * G * kHeadDim + e] = acc;
    }
  return HCA_OK;
}
