// One decode step through the C ABI with no PyTorch anywhere: device memory from hipMalloc, the value store
// from hipHostMalloc, inputs from a small linear congruential generator, the result checked against the CPU
// oracle (linked as a shared object).  Built with hipcc and run by tests/test_gpu_parity.py.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "hca.h"

extern "C" {
int hco_quantize(const uint16_t* k_new, int64_t R, int64_t T, int D, int bits, int gs, int64_t cap, const int64_t* n0,
                 uint8_t* codes, uint16_t* scale, uint16_t* zero);
int hco_score(const uint16_t* q, const uint8_t* codes, const uint16_t* scale, const uint16_t* zero, int64_t R, int G,
              int D, int bits, int gs, int64_t cap, const int64_t* n, float* sel, float* z);
int hco_topk(const float* sel, int64_t R, int64_t cap, const int64_t* n, int64_t k, int32_t* idx, int32_t* count);
int hco_attend(const uint16_t* q, const uint8_t* codes, const uint16_t* scale, const uint16_t* zero, int64_t R, int G,
               int D, int bits, int gs, int64_t cap, const int32_t* idx, const int32_t* count, int64_t k,
               const int32_t* pos, const uint16_t* V, int64_t vrows, float sm_scale, float* y, float* w_opt,
               float* acc_opt, const float* lse_opt);
}

#define HIP_OK(x)                                                                        \
  do {                                                                                   \
    hipError_t e_ = (x);                                                                 \
    if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 2; } \
  } while (0)
#define HCA_OK_(x)                                                             \
  do {                                                                         \
    int32_t r_ = (x);                                                          \
    if (r_ != HCA_OK) { printf("hca error %d at line %d\n", r_, __LINE__); return 3; } \
  } while (0)

static uint64_t lcg_state = 0x9E3779B97F4A7C15ull;
static float uniform() {   // (-1, 1)
  lcg_state = lcg_state * 6364136223846793005ull + 1442695040888963407ull;
  return (float)((lcg_state >> 40) & 0xffffff) / 8388608.0f - 1.0f;
}
static uint16_t to_half(float x) {
  _Float16 h = (_Float16)x;
  uint16_t b;
  std::memcpy(&b, &h, 2);
  return b;
}

int main() {
  const int batch = 2, hkv = 2, G = 4, D = 128, bits = 4, gs = 32, k = 96;
  const int64_t n = 3001, cap = 3010, R = batch * hkv;
  std::vector<uint16_t> keys((size_t)R * n * D), vals((size_t)R * n * D), q((size_t)R * G * D);
  for (auto& x : keys) x = to_half(2.0f * uniform());
  for (auto& x : vals) x = to_half(uniform());
  for (int64_t hq = 0; hq < R * G; ++hq)          // each query resembles one of its row's keys
    for (int c = 0; c < D; ++c) {
      const int64_t r = hq / G, j = (hq * 397 + 11) % n;
      _Float16 kv;
      std::memcpy(&kv, &keys[((size_t)r * n + j) * D + c], 2);
      q[(size_t)hq * D + c] = to_half((float)kv + 0.2f * uniform());
    }

  hca_shape s = {batch, hkv * G, hkv, D, bits, gs, cap};
  void *kc, *dk, *dq, *ws, *vh;
  float *sel, *y, *acc;
  int32_t *idx, *count, *pos;
  HIP_OK(hipMalloc(&kc, hca_kcache_bytes(&s)));
  HIP_OK(hipMalloc(&dk, keys.size() * 2));
  HIP_OK(hipMalloc(&dq, q.size() * 2));
  HIP_OK(hipMalloc(&ws, hca_workspace_bytes(&s, k, 1)));
  HIP_OK(hipMalloc(&sel, (size_t)R * cap * 4));
  HIP_OK(hipMalloc(&y, (size_t)R * G * D * 4));
  HIP_OK(hipMalloc(&acc, (size_t)R * cap * 4));
  HIP_OK(hipMalloc(&idx, (size_t)R * k * 4));
  HIP_OK(hipMalloc(&count, (size_t)R * 4));
  HIP_OK(hipMalloc(&pos, (size_t)R * cap * 4));
  HIP_OK(hipHostMalloc(&vh, vals.size() * 2, hipHostMallocDefault));
  std::memcpy(vh, vals.data(), vals.size() * 2);
  HIP_OK(hipMemcpy(dk, keys.data(), keys.size() * 2, hipMemcpyHostToDevice));
  HIP_OK(hipMemcpy(dq, q.data(), q.size() * 2, hipMemcpyHostToDevice));
  HIP_OK(hipMemset(acc, 0, (size_t)R * cap * 4));
  hipStream_t st, gst;
  HIP_OK(hipStreamCreate(&st));
  HIP_OK(hipStreamCreate(&gst));

  int64_t n0[2] = {0, 0}, nres[2] = {n, n}, row0[2] = {0, 0};
  const float sm = 1.0f / std::sqrt((float)D);
  HCA_OK_(hca_quantize_keys(&s, kc, dk, n, n0, acc, pos, row0, st));
  HCA_OK_(hca_score_qkeys(&s, kc, dq, nres, sel, nullptr, nullptr, st));
  HCA_OK_(hca_topk(&s, sel, nres, k, idx, count, ws, st));
  HCA_OK_(hca_sparse_attend(&s, kc, dq, idx, count, k, pos, vh, n, n, nullptr, 0, sm, y, acc, ws, gst, st));
  // the same selection as one call that writes no per-token scores
  int32_t *fidx, *fcount;
  HIP_OK(hipMalloc(&fidx, (size_t)R * k * 4));
  HIP_OK(hipMalloc(&fcount, (size_t)R * 4));
  HCA_OK_(hca_score_topk(&s, kc, dq, nres, k, fidx, fcount, ws, st));
  HIP_OK(hipStreamSynchronize(st));

  std::vector<int32_t> gidx((size_t)R * k), gcount(R);
  std::vector<float> gy((size_t)R * G * D), gacc((size_t)R * cap);
  std::vector<int32_t> fgidx((size_t)R * k), fgcount(R);
  HIP_OK(hipMemcpy(fgidx.data(), fidx, fgidx.size() * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(fgcount.data(), fcount, fgcount.size() * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(gidx.data(), idx, gidx.size() * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(gcount.data(), count, gcount.size() * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(gy.data(), y, gy.size() * 4, hipMemcpyDeviceToHost));
  HIP_OK(hipMemcpy(gacc.data(), acc, gacc.size() * 4, hipMemcpyDeviceToHost));

  // the oracle on the same inputs
  std::vector<uint8_t> codes((size_t)R * cap * D * bits / 8);
  std::vector<uint16_t> scale((size_t)R * cap * (D / gs)), zero(scale.size());
  std::vector<int64_t> on0(R, 0), on(R, n);
  std::vector<float> osel((size_t)R * cap, 0.f), oy((size_t)R * G * D), oacc((size_t)R * cap, 0.f);
  std::vector<int32_t> oidx((size_t)R * k), ocount(R), opos((size_t)R * cap);
  for (int64_t r = 0; r < R; ++r)
    for (int64_t j = 0; j < cap; ++j) opos[(size_t)r * cap + j] = (int32_t)j;
  if (hco_quantize(keys.data(), R, n, D, bits, gs, cap, on0.data(), codes.data(), scale.data(), zero.data())) return 4;
  if (hco_score(q.data(), codes.data(), scale.data(), zero.data(), R, G, D, bits, gs, cap, on.data(), osel.data(), nullptr)) return 4;
  if (hco_topk(osel.data(), R, cap, on.data(), k, oidx.data(), ocount.data())) return 4;
  if (hco_attend(q.data(), codes.data(), scale.data(), zero.data(), R, G, D, bits, gs, cap, oidx.data(), ocount.data(), k,
                 opos.data(), vals.data(), n, sm, oy.data(), nullptr, oacc.data(), nullptr)) return 4;

  for (int64_t r = 0; r < R; ++r) {
    if (gcount[r] != ocount[r] || gcount[r] != k) { printf("count differs in row %ld\n", (long)r); return 5; }
    for (int i = 0; i < k; ++i)
      if (gidx[(size_t)r * k + i] != oidx[(size_t)r * k + i]) { printf("top-k differs in row %ld\n", (long)r); return 5; }
    if (fgcount[r] != ocount[r]) { printf("fused count differs in row %ld\n", (long)r); return 5; }
    for (int i = 0; i < k; ++i)
      if (fgidx[(size_t)r * k + i] != oidx[(size_t)r * k + i]) { printf("fused top-k differs in row %ld\n", (long)r); return 5; }
  }
  double worst = 0.0;
  for (int64_t hq = 0; hq < R * G; ++hq) {
    double num = 0.0, den = 1e-30;
    for (int c = 0; c < D; ++c) {
      num = std::fmax(num, std::fabs((double)gy[(size_t)hq * D + c] - oy[(size_t)hq * D + c]));
      den = std::fmax(den, std::fabs((double)oy[(size_t)hq * D + c]));
    }
    worst = std::fmax(worst, num / den);
  }
  if (worst > 2e-3) { printf("output differs: %g\n", worst); return 6; }
  for (size_t i = 0; i < gacc.size(); ++i)
    if (std::fabs(gacc[i] - oacc[i]) > 1e-4f * std::fabs(oacc[i]) + 1e-7f) { printf("acc differs at %zu\n", i); return 7; }
  printf("decode step without torch ok: top-k sets exact, output rel err %.3g\n", worst);
  return 0;
}
