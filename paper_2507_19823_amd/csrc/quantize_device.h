// Device side of the key quantisation (the compressor Q(K) of Eq. 2 in scale/zero form), shared by the
// append kernel and by kernels that append one token beside other work.
#pragma once
#include "hca_device.h"

namespace hca {

// One wave quantises 16 tokens.  Lane (t = lane%16, j = lane/16) owns the two 16-channel
// pieces of token t that it will later feed to the matrix core (see Layout), i.e. input bytes
// [32j, 32j+32) and [128+32j, 128+32j+32) of the token's 256-byte fp16 row.
// bx = index of the workgroup's 64 tokens, n_before = the row's resident slots, vrow0 = value row of the first new
// token; called by all 256 threads of a workgroup.
template <int BITS>
__device__ __forceinline__ void quantize_body(const Layout& L, uint8_t* __restrict__ kcache,
                                              const uint16_t* __restrict__ k_new, int64_t T, const int64_t n_before,
                                              float* __restrict__ acc, int32_t* __restrict__ pos, const int64_t vrow0,
                                              const int bx, const int row) {
  constexpr int QMAX = (1 << BITS) - 1;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int t = lane & 15, j = lane >> 4;
  const int64_t tt = ((int64_t)bx * 4 + w) * 16 + t;
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
    // x >= mn, so the quotient is never negative: one upper clamp, then the saturating float -> byte
    // conversion, which rounds to nearest even and drops the code into its byte of a dword (4 codes each).
    uint32_t b[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float v = fminf((x[m][i] - mn) * inv, (float)QMAX);
      b[i >> 2] = __builtin_amdgcn_cvt_pk_u8_f32(v, (uint32_t)(i & 3), b[i >> 2]);
    }
    // bytes -> packed codes: even- and odd-numbered codes of two dwords gathered bytewise, the odd ones
    // shifted up by one code width; once for 4-bit codes, twice for 2-bit codes
    constexpr uint32_t kEven = 0x06040200u, kOdd = 0x07050301u;
    uint32_t lo = __builtin_amdgcn_perm(b[1], b[0], kEven) | (__builtin_amdgcn_perm(b[1], b[0], kOdd) << BITS);
    uint32_t hi = __builtin_amdgcn_perm(b[3], b[2], kEven) | (__builtin_amdgcn_perm(b[3], b[2], kOdd) << BITS);
    if (BITS == 2) {
      lo = __builtin_amdgcn_perm(hi, lo, kEven) | (__builtin_amdgcn_perm(hi, lo, kOdd) << 4);
      hi = 0;
    }
    packed[m][0] = lo;
    packed[m][1] = hi;
    meta[m] = (uint32_t)sh | ((uint32_t)f2h_bits(mn) << 16);
  }

  const int64_t slot = n_before + tc;
  uint8_t* crow = kcache + (int64_t)row * L.codes_row_bytes();
  uint8_t* mrow = kcache + L.meta_off + (int64_t)row * L.meta_row_bytes();
  if (live && j == 1 && acc != nullptr) acc[(int64_t)row * L.cap + slot] = 0.0f;
  if (live && j == 2 && pos != nullptr) pos[(int64_t)row * L.cap + slot] = (int32_t)(vrow0 + tt);
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

}  // namespace hca
