// Step 1: key quantisation and append (the compressor Q(K) of Eq. 2 in scale/zero form),
// plus the canonical export used by tests.
#include "hca_internal.h"

namespace hca {

// One wave quantises 16 tokens.  Lane (t = lane%16, j = lane/16) owns the two 16-channel
// pieces of token t that it will later feed to the matrix core (see Layout), i.e. input bytes
// [32j, 32j+32) and [128+32j, 128+32j+32) of the token's 256-byte fp16 row.
template <int BITS>
__global__ __launch_bounds__(256) void quantize_kernel(Layout L, uint8_t* __restrict__ kcache,
                                                       const uint16_t* __restrict__ k_new, int64_t T, NRes nr,
                                                       float* __restrict__ acc, int32_t* __restrict__ pos, NRes vrow0) {
  constexpr int QMAX = (1 << BITS) - 1;
  const int row = blockIdx.y;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int t = lane & 15, j = lane >> 4;
  const int64_t tt = ((int64_t)blockIdx.x * 4 + w) * 16 + t;
  const bool live = tt < T;
  const int64_t tc = live ? tt : T - 1;
  const uint4* src = reinterpret_cast<const uint4*>(k_new + ((int64_t)row * T + tc) * kHeadDim);
  uint4 raw[2][2];
  raw[0][0] = src[2 * j];
  raw[0][1] = src[2 * j + 1];
  raw[1][0] = src[8 + 2 * j];
  raw[1][1] = src[8 + 2 * j + 1];

  float x[2][16];
#pragma unroll
  for (int m = 0; m < 2; ++m)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t wds[4] = {raw[m][h].x, raw[m][h].y, raw[m][h].z, raw[m][h].w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        x[m][8 * h + 2 * i] = h2f(wds[i] & 0xffffu);
        x[m][8 * h + 2 * i + 1] = h2f(wds[i] >> 16);
      }
    }

  uint32_t packed[2][2];
  uint32_t meta[2];  // scale bits | zero bits << 16, per slot m
#pragma unroll
  for (int m = 0; m < 2; ++m) {
    float mn = x[m][0], mx = x[m][0];
#pragma unroll
    for (int i = 1; i < 16; ++i) { mn = fminf(mn, x[m][i]); mx = fmaxf(mx, x[m][i]); }
    mn = fminf(mn, __shfl_xor(mn, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    if (BITS == 2) {  // a 64-channel group spans all four lanes of the token
      mn = fminf(mn, __shfl_xor(mn, 32));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
    }
    if (mn == 0.0f) mn = 0.0f;  // -0 -> +0
    const float range = mx - mn;
    unsigned short sh = f2h_bits(range / (float)QMAX);
    if ((sh & 0x7fffu) == 0) sh = 0x3c00u;
    const float sc = h2f(sh);
    const float inv = 1.0f / sc;
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      float v = rintf((x[m][i] - mn) * inv);
      v = fminf(fmaxf(v, 0.0f), (float)QMAX);
      const uint32_t c = (uint32_t)(int)v;
      if (BITS == 4) {
        if (i < 8) lo |= c << (4 * i); else hi |= c << (4 * (i - 8));
      } else {
        lo |= c << (2 * i);
      }
    }
    packed[m][0] = lo;
    packed[m][1] = hi;
    meta[m] = (uint32_t)sh | ((uint32_t)f2h_bits(mn) << 16);
  }

  const int64_t slot = nr.n[row / L.n_kv_heads] + tc;
  uint8_t* crow = kcache + (int64_t)row * L.codes_row_bytes();
  uint8_t* mrow = kcache + L.meta_off + (int64_t)row * L.meta_row_bytes();
  if (live && j == 1 && acc != nullptr) acc[(int64_t)row * L.cap + slot] = 0.0f;
  if (live && j == 2 && pos != nullptr) pos[(int64_t)row * L.cap + slot] = (int32_t)(vrow0.n[row / L.n_kv_heads] + tt);
  if (BITS == 4) {
    const uint32_t o0 = __shfl_xor(meta[0], 32), o1 = __shfl_xor(meta[1], 32);
    if (live) {
      const int64_t blk = slot >> 4;
      const int tl = (int)(slot & 15);
      *reinterpret_cast<uint4*>(crow + blk * kBlockBytes + (tl + 16 * j) * 16) =
          uint4{packed[0][0], packed[0][1], packed[1][0], packed[1][1]};
      if (j == 0) {  // own: groups 0 (m=0), 2 (m=1); partner lane j=2: groups 1, 3
        uint4 mw;
        mw.x = (meta[0] & 0xffffu) | (o0 << 16);
        mw.y = (meta[1] & 0xffffu) | (o1 << 16);
        mw.z = (meta[0] >> 16) | (o0 & 0xffff0000u);
        mw.w = (meta[1] >> 16) | (o1 & 0xffff0000u);
        *reinterpret_cast<uint4*>(mrow + blk * kMetaBytes + tl * 16) = mw;
      }
    }
  } else {
    if (live) {
      const int64_t blk = slot >> 5;
      const int u = (int)((slot >> 4) & 1), tl = (int)(slot & 15);
      *reinterpret_cast<uint2*>(crow + blk * kBlockBytes + (tl + 16 * j) * 16 + 8 * u) =
          uint2{packed[0][0], packed[1][0]};
      if (j == 0) {
        uint2 mw;
        mw.x = (meta[0] & 0xffffu) | (meta[1] << 16);
        mw.y = (meta[0] >> 16) | (meta[1] & 0xffff0000u);
        *reinterpret_cast<uint2*>(mrow + blk * kMetaBytes + (16 * u + tl) * 8) = mw;
      }
    }
  }
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
