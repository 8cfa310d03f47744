// Step 1: key quantisation and append (the compressor Q(K) of Eq. 2 in scale/zero form),
// plus the canonical export used by tests.
#include "hca_internal.h"
#include "quantize_device.h"

namespace hca {

template <int BITS>
__global__ __launch_bounds__(256) void quantize_kernel(Layout L, uint8_t* __restrict__ kcache,
                                                       const uint16_t* __restrict__ k_new, int64_t T, NRes nr,
                                                       float* __restrict__ acc, int32_t* __restrict__ pos, NRes vrow0) {
  const int seq = blockIdx.y / L.n_kv_heads;
  quantize_body<BITS>(L, kcache, k_new, T, nr.n[seq], acc, pos, vrow0.n[seq], (int)blockIdx.x, (int)blockIdx.y);
}

// Canonical export: one thread per (slot, j) piece.
template <int BITS>
__global__ __launch_bounds__(256) void export_kernel(Layout L, const uint8_t* __restrict__ kcache, NRes nr,
                                                     uint8_t* __restrict__ codes, uint16_t* __restrict__ scale,
                                                     uint16_t* __restrict__ zero) {
  const int row = blockIdx.y;
  const int64_t n = nr.n[row / L.n_kv_heads];
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t slot = gid >> 2;
  const int j = (int)(gid & 3);
  if (slot >= n) return;
  const uint8_t* crow = kcache + (int64_t)row * L.codes_row_bytes();
  const uint8_t* mrow = kcache + L.meta_off + (int64_t)row * L.meta_row_bytes();
  constexpr int CB = kHeadDim * BITS / 8;
  uint8_t* out = codes + ((int64_t)row * L.cap + slot) * CB;
  uint16_t* so = scale + ((int64_t)row * L.cap + slot) * L.ng;
  uint16_t* zo = zero + ((int64_t)row * L.cap + slot) * L.ng;
  if (BITS == 4) {
    const int64_t blk = slot >> 4;
    const int tl = (int)(slot & 15);
    const uint4 w = *reinterpret_cast<const uint4*>(crow + blk * kBlockBytes + (tl + 16 * j) * 16);
    // slot m covers channels [32(2m + j/2) + 16(j%2), +16) -> canonical bytes at half that offset
    uint2* o0 = reinterpret_cast<uint2*>(out + (32 * (0 + (j >> 1)) + 16 * (j & 1)) / 2);
    uint2* o1 = reinterpret_cast<uint2*>(out + (32 * (2 + (j >> 1)) + 16 * (j & 1)) / 2);
    *o0 = uint2{w.x, w.y};
    *o1 = uint2{w.z, w.w};
    if (j == 0) {
      const uint4 mw = *reinterpret_cast<const uint4*>(mrow + blk * kMetaBytes + tl * 16);
      so[0] = mw.x & 0xffffu; so[1] = mw.x >> 16; so[2] = mw.y & 0xffffu; so[3] = mw.y >> 16;
      zo[0] = mw.z & 0xffffu; zo[1] = mw.z >> 16; zo[2] = mw.w & 0xffffu; zo[3] = mw.w >> 16;
    }
  } else {
    const int64_t blk = slot >> 5;
    const int u = (int)((slot >> 4) & 1), tl = (int)(slot & 15);
    const uint2 w = *reinterpret_cast<const uint2*>(crow + blk * kBlockBytes + (tl + 16 * j) * 16 + 8 * u);
    *reinterpret_cast<uint32_t*>(out + (64 * 0 + 16 * j) / 4) = w.x;
    *reinterpret_cast<uint32_t*>(out + (64 * 1 + 16 * j) / 4) = w.y;
    if (j == 0) {
      const uint2 mw = *reinterpret_cast<const uint2*>(mrow + blk * kMetaBytes + (16 * u + tl) * 8);
      so[0] = mw.x & 0xffffu; so[1] = mw.x >> 16;
      zo[0] = mw.y & 0xffffu; zo[1] = mw.y >> 16;
    }
  }
}

int32_t launch_quantize(const Layout& L, void* kcache, const void* k_new, int64_t T, const NRes& nr,
                        float* acc_opt, int32_t* pos_opt, const NRes& vrow0, hipStream_t st) {
  if (T == 0) return HCA_OK;
  dim3 grid((unsigned)((T + 63) / 64), (unsigned)L.rows);
  if (L.bits == 4)
    quantize_kernel<4><<<grid, 256, 0, st>>>(L, (uint8_t*)kcache, (const uint16_t*)k_new, T, nr, acc_opt, pos_opt, vrow0);
  else
    quantize_kernel<2><<<grid, 256, 0, st>>>(L, (uint8_t*)kcache, (const uint16_t*)k_new, T, nr, acc_opt, pos_opt, vrow0);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

int32_t launch_export(const Layout& L, const void* kcache, const NRes& nr, uint8_t* codes, void* scale,
                      void* zero, hipStream_t st) {
  int64_t nmax = 0;
  for (int b = 0; b < L.batch; ++b) nmax = nr.n[b] > nmax ? nr.n[b] : nmax;
  if (nmax == 0) return HCA_OK;
  dim3 grid((unsigned)((nmax * 4 + 255) / 256), (unsigned)L.rows);
  if (L.bits == 4)
    export_kernel<4><<<grid, 256, 0, st>>>(L, (const uint8_t*)kcache, nr, codes, (uint16_t*)scale, (uint16_t*)zero);
  else
    export_kernel<2><<<grid, 256, 0, st>>>(L, (const uint8_t*)kcache, nr, codes, (uint16_t*)scale, (uint16_t*)zero);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

}  // namespace hca
