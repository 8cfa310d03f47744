/* The boundary from plain C: include/hca.h must compile as C11, every entry point must link from
 * libhca.so, and the host-side validation must work without a GPU.  Built and run by
 * tests/test_abi_host.py (gcc, no HIP headers, no torch). */
#include <stdio.h>
#include <string.h>

#include "hca.h"

#define CHECK(cond)                                                   \
  do {                                                                \
    if (!(cond)) {                                                    \
      printf("FAILED line %d: %s\n", __LINE__, #cond);                \
      return 1;                                                       \
    }                                                                 \
  } while (0)

int main(void) {
  hca_shape s;
  memset(&s, 0, sizeof s);
  s.batch = 1; s.n_q_heads = 32; s.n_kv_heads = 8; s.head_dim = 128; s.bits = 4; s.group = 32;
  s.capacity = 1 << 20;
  CHECK(strncmp(hca_version(), "hca", 3) == 0);
  CHECK(hca_kcache_bytes(&s) == (size_t)8 * (1 << 20) * 80);
  CHECK(hca_workspace_bytes(&s, 4096, 1 << 20) > 0);
  CHECK(hca_tune("gather_unroll", 4) == HCA_OK);
  CHECK(hca_tune("nonsense", 1) == HCA_ERR_BAD_ARG);

  int64_t n[1] = {100};
  char dummy[256];
  void* p = dummy;                      /* never dereferenced: validation fails first */
  CHECK(hca_quantize_keys(&s, NULL, p, 1, n, NULL, NULL, NULL, NULL) == HCA_ERR_BAD_ARG);
  CHECK(hca_score_qkeys(&s, p, p, NULL, (float*)p, NULL, NULL, NULL) == HCA_ERR_BAD_ARG);
  CHECK(hca_topk(&s, (const float*)p, n, 0, (int32_t*)p, (int32_t*)p, p, NULL) == HCA_ERR_CAPACITY);
  CHECK(hca_score_topk(&s, p, p, n, 0, (int32_t*)p, (int32_t*)p, p, NULL) == HCA_ERR_CAPACITY);
  CHECK(hca_topp(&s, (const float*)p, n, 0.1f, 0.0, 8, (int32_t*)p, (int32_t*)p, NULL, p, NULL) == HCA_ERR_BAD_ARG);
  CHECK(hca_evict(&s, p, (float*)p, (int32_t*)p, n, 0, 0, NULL, p, NULL, NULL, NULL, NULL) == HCA_ERR_CAPACITY);
  s.bits = 3;
  CHECK(hca_kcache_bytes(&s) == 0);
  CHECK(hca_score_qkeys(&s, p, p, n, (float*)p, NULL, NULL, NULL) == HCA_ERR_UNSUPPORTED);
  s.bits = 4;

  hca_vq_codebook cb;
  cb.groups = 32; cb.codewords = 256; cb.centroids = NULL;
  CHECK(hca_vq_pcache_bytes(&s, &cb) == (size_t)8 * (1 << 20) * 32);
  CHECK(hca_vq_lut_bytes(&s, &cb) == (size_t)8 * 32 * 256 * 4 * 4 + 8 * 33 * 4 * 4);
  CHECK(hca_vq_assign(&s, &cb, p, p, 1, n, NULL, NULL, NULL, NULL) == HCA_ERR_BAD_ARG);   /* no centroids */

  /* the host-side trainer runs anywhere: two well separated points per group, two centroids */
  unsigned short kval[4 * 128];
  for (int t = 0; t < 4; ++t)
    for (int c = 0; c < 128; ++c) kval[t * 128 + c] = (t < 2) ? 0x3c00 /* 1.0 */ : 0xc400 /* -4.0 */;
  int32_t init[32 * 2];
  for (int i = 0; i < 32; ++i) { init[2 * i] = 0; init[2 * i + 1] = 3; }
  float cen[32 * 2 * 4];
  double inertia[3];
  CHECK(hca_vq_train(kval, 4, 128, 32, 2, init, 2, 0, cen, inertia) == HCA_OK);
  CHECK(cen[0] == 1.0f && cen[4] == -4.0f && inertia[2] == 0.0);

  CHECK(hca_pipeline_create(&s, 0, NULL, 0) == NULL);
  printf("abi ok: %s\n", hca_version());
  return 0;
}
