// Codebook form of the key path: grouped vector quantisation (Sec. 3.1) and the table-lookup
// scores of Sec. 3.2, Eq. 3.  A token is one centroid index per group (a byte: c <= 256), the query
// becomes a table T[centroid][group][query head of the KV head] that sits in LDS while a workgroup
// scans its share of the index matrix.  The host-side trainer is at the end of the file.
//
// Two storage forms.  Narrow (c <= 256 and the table of a KV head within 128 KiB): byte indices, table in
// LDS - everything said above.  Wide (up to c = 8192, the paper's own size, Fig. 4 / Table 4a): 16-bit
// indices stored group-major in tiles of 16 Ki slots (vq_wide_at in hca_device.h) and a table kept
// group-major too; a workgroup scans one tile and brings the table through LDS one slice of groups at a
// time (vq_scan_wide_kernel).
//
// Narrow index rows are stored rotated: byte p of the record of slot j holds the index of group
// 16 * (p / 16) + (p + j) % 16  (vq_byte_of / vq_group_at in hca_device.h).  A thread of the scan reads
// its token's bytes in storage order, so at any moment the 16 lanes that share one pass of a 16-byte
// LDS read are on 16 different groups, and because a group's entries sit 16 bytes apart within a
// centroid's 256-byte line those lanes hit 16 different sets of 4 banks whatever their indices are.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <thread>
#include <vector>

#include "hca_internal.h"

namespace hca {

// ------------------------------------------------------------------------------- assign ---
// One wave = 64 tokens x GPW consecutive groups (4 for bulk calls; 1 for blocks of a few thousand tokens, which
// would otherwise leave most of the chip without a wave).  Every centroid read is wave-uniform (scalar loads),
// the running minimum is per lane.  distance: e = x - c; d = fmaf(e, e, d) over the group's channels in ascending
// order from d = 0; the first smallest wins.
template <int DBAR, bool WIDE, int GPW>
__global__ __launch_bounds__(256) void vq_assign_kernel(int g, int c, int n_kv_heads, int64_t cap,
                                                        const float* __restrict__ centroids,
                                                        uint8_t* __restrict__ pcache, const uint16_t* __restrict__ k_new,
                                                        int64_t T, NRes nr, float* __restrict__ acc,
                                                        int32_t* __restrict__ pos, NRes vrow0) {
  const int row = blockIdx.y;
  const int lane = threadIdx.x & 63;
  const int g0 = __builtin_amdgcn_readfirstlane((int)(blockIdx.z * 4 + (threadIdx.x >> 6))) * GPW;   // first group
  if (g0 >= g) return;
  const int64_t tt = (int64_t)blockIdx.x * 64 + lane;
  const bool live = tt < T;
  const int64_t tc = live ? tt : T - 1;
  // the wave's GPW * DBAR channels of this lane's token
  float x[GPW][DBAR];
  {
    const uint16_t* src = k_new + ((int64_t)row * T + tc) * kHeadDim + g0 * DBAR;
    constexpr int NW32 = GPW * DBAR / 2;                  // dwords: 8, 4, 2 or 1
    uint32_t wd[NW32];
    if constexpr (NW32 == 8) {
      const uint4 a = reinterpret_cast<const uint4*>(src)[0], b = reinterpret_cast<const uint4*>(src)[1];
      wd[0] = a.x; wd[1] = a.y; wd[2] = a.z; wd[3] = a.w; wd[4] = b.x; wd[5] = b.y; wd[6] = b.z; wd[7] = b.w;
    } else if constexpr (NW32 == 4) {
      const uint4 a = reinterpret_cast<const uint4*>(src)[0];
      wd[0] = a.x; wd[1] = a.y; wd[2] = a.z; wd[3] = a.w;
    } else if constexpr (NW32 == 2) {
      const uint2 a = reinterpret_cast<const uint2*>(src)[0];
      wd[0] = a.x; wd[1] = a.y;
    } else {
      wd[0] = reinterpret_cast<const uint32_t*>(src)[0];
    }
#pragma unroll
    for (int i = 0; i < NW32; ++i) {
      const int ch = 2 * i;
      x[ch / DBAR][ch % DBAR] = h2f(wd[i] & 0xffffu);
      x[(ch + 1) / DBAR][(ch + 1) % DBAR] = h2f(wd[i] >> 16);
    }
  }
  const float* cb = centroids + ((int64_t)(row % n_kv_heads) * g + g0) * c * DBAR;
  int win[GPW];
#pragma unroll
  for (int u = 0; u < GPW; ++u) {
    const float* cg = cb + (int64_t)u * c * DBAR;
    float bd = INFINITY;
    int best = 0;
    for (int cc = 0; cc < c; ++cc) {
      float d = 0.f;
#pragma unroll
      for (int dd = 0; dd < DBAR; ++dd) {
        const float e = x[u][dd] - cg[cc * DBAR + dd];
        d = fmaf(e, e, d);
      }
      if (d < bd || cc == 0) { bd = d; best = cc; }
    }
    win[u] = best;
  }
  if (!live) return;
  const int b = row / n_kv_heads;
  const int64_t slot = nr.n[b] + tt;
  if constexpr (WIDE) {
    uint16_t* pw = reinterpret_cast<uint16_t*>(pcache);
    const int64_t tiles = vq_tiles(cap);
#pragma unroll
    for (int u = 0; u < GPW; ++u) pw[vq_wide_at(g, tiles, row, slot, g0 + u)] = (uint16_t)win[u];
  } else {
    uint8_t* rec = pcache + ((int64_t)row * cap + slot) * g;
#pragma unroll
    for (int u = 0; u < GPW; ++u) rec[vq_byte_of(g0 + u, slot)] = (uint8_t)win[u];
  }
  if (g0 == 0) {
    if (acc != nullptr) acc[(int64_t)row * cap + slot] = 0.0f;
    if (pos != nullptr) pos[(int64_t)row * cap + slot] = (int32_t)(vrow0.n[b] + tt);
  }
}

// Bulk calls (a prefill block, a whole context): the matrix cores find, for every token, the few centroids that can
// be the nearest one, and only those go through the exact distance chain of vq_assign_kernel - the same index, bit
// for bit.
//   e(c) = |c|^2 / 2 - x.c  (= (distance - |x|^2) / 2) comes out of v_mfma_f32_32x32x16_f16, 32 centroids x 32 tokens
//   per instruction, with every factor an fp16 number so that the 16 products are exact in fp32:
//     k 0..3   A = -hi(c_d)            B = x_d        hi(c) = fp16(c), lo(c) = fp16(c - hi(c))
//     k 4..7   A = -lo(c_d)            B = x_d        (x is fp16 as it arrives)
//     k 8..10  A = h1, h2, h3          B = 1          h = fp32 |c|^2 / 2 cut into three fp16 pieces
//     k 11..13 A = 1                   B = t1, t2, t3 pass 2 only: t = -(threshold) in three fp16 pieces
//   Errors against the exact e(c), with S = |x|^2 + max_c |c|^2 < 2^15 (so that no piece overflows fp16; fp16
//   denormals are kept by the instruction): c_d - hi - lo is at most 2^-22 |c_d| + 2^-25, h and t lose at most
//   2^-33 of themselves + 2^-25, the fp32 |c|^2 chain 4 u |c|^2 (u = 2^-24), and the instruction's 15 additions at
//   most 2^-23 each of sum |terms| <= 2.01 S whatever their order and rounding: together below 2^-17.9 S + 2^-23.
//   The exact chain d(c) itself is within 7 u d <= 2^-20.2 S of the truth (in units of e).  With
//   delta = 2^-16 S + 2^-21 - three times the sum of those - the winner c* of the exact chain (first smallest d)
//   has e(c*) - (min_c e(c) + 2 delta) < 0 as computed in pass 2.
//   Pass 1 takes min_c e(c) per token (eight v_min3 per instruction).  Pass 2 runs the same products with the
//   threshold folded in and collects the sign bits (eight v_or3): a centroid whose result is negative is noted
//   in the lane's candidate list - one or two per token; a candidate that finds the list full goes through the
//   exact chain at once and only the best of those is kept.  Then the exact chain runs over the list in ascending
//   index order.  A token whose S is out of range or not a number takes the exact chain over every centroid
//   instead (same result, the speed of the vector form).
// One workgroup of 8 waves = 1024 tokens x one group; a wave holds 128 tokens (four 32-token B operands) against
// centroids that pass through LDS 512 at a time (A operands only, double-buffered, one barrier per chunk).
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
constexpr int kAmChunk = 512;       // centroids per LDS chunk
// the matrix-core form is taken from 1024 tokens x 2048 centroids (or 4096 x 512) on: level with the vector forms
// at 256 centroids, ahead of them from 512 on, and a workgroup wants 1024 tokens
constexpr int64_t kAssignMfmaMinTokens = 1024;
constexpr int kAssignMfmaMinCodewords = 512;
constexpr int64_t kAssignMfmaMinWork = (int64_t)1 << 21;
constexpr int kAmCand = 3;          // candidate slots per lane (two lanes per token); further ones are judged at once

__device__ __forceinline__ _Float16 am_f16(float v) { return (_Float16)v; }

template <int DBAR, bool WIDE>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(4))) void vq_assign_mfma_kernel(
    int g, int c, int n_kv_heads, int64_t cap, const float* __restrict__ centroids, uint8_t* __restrict__ pcache,
    const uint16_t* __restrict__ k_new, int64_t T, NRes nr, float* __restrict__ acc, int32_t* __restrict__ pos,
    NRes vrow0) {
  // A operands: [buffer][tile of 32 centroids][k block 0 / 1][row] x 8 fp16
  __shared__ __align__(16) v8h sA[2][kAmChunk / 32][2][32];
  __shared__ float s_cmax[8];
  const int row = blockIdx.y, grp = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int col = lane & 31, kb = lane >> 5;
  const int64_t tok0 = (int64_t)blockIdx.x * 1024 + w * 128;
  const float* cg = centroids + ((int64_t)(row % n_kv_heads) * g + grp) * c * DBAR;

  // this lane's tokens: |x|^2 and the B operand of its k block (x itself is read again for the exact chain)
  float x2[4];
  v8h bop[4];
#pragma unroll
  for (int tt = 0; tt < 4; ++tt) {
    const int64_t t = tok0 + 32 * tt + col;
    const int64_t tc = t < T ? t : T - 1;
    const uint16_t* src = k_new + ((int64_t)row * T + tc) * kHeadDim + grp * DBAR;
    float n2 = 0.f;
    _Float16 xh[4] = {(_Float16)0.f, (_Float16)0.f, (_Float16)0.f, (_Float16)0.f};
#pragma unroll
    for (int d = 0; d < DBAR; ++d) {
      const uint16_t bits = src[d];
      const float xf = h2f(bits);
      xh[d] = __builtin_bit_cast(_Float16, bits);
      n2 = fmaf(xf, xf, n2);
    }
    x2[tt] = n2;
    const _Float16 one = (_Float16)1.f, zero = (_Float16)0.f;
    if (kb == 0) bop[tt] = v8h{xh[0], xh[1], xh[2], xh[3], xh[0], xh[1], xh[2], xh[3]};
    else bop[tt] = v8h{one, one, one, zero, zero, zero, zero, zero};
  }

  const int nchunk = (c + kAmChunk - 1) / kAmChunk;
  v8h ra0, ra1;                      // this thread's centroid of the chunk on its way to LDS
  float rn = 0.f;
  auto fetch = [&](int ch) {
    const int cc = ch * kAmChunk + tid;
    const _Float16 one = (_Float16)1.f, zero = (_Float16)0.f;
    ra0 = v8h{zero, zero, zero, zero, zero, zero, zero, zero};
    ra1 = v8h{(_Float16)65504.f, zero, zero, one, one, one, zero, zero};     // past the codebook: never the minimum
    rn = 0.f;
    if (cc < c) {
      float nn = 0.f;
      _Float16 hi[4] = {zero, zero, zero, zero}, lo[4] = {zero, zero, zero, zero};
#pragma unroll
      for (int d = 0; d < DBAR; ++d) {
        const float v = cg[(int64_t)cc * DBAR + d];
        nn = fmaf(v, v, nn);
        hi[d] = am_f16(-v);
        lo[d] = am_f16(-v - (float)hi[d]);
      }
      const float hh = 0.5f * nn;
      const _Float16 h1 = am_f16(hh);
      const float r1 = hh - (float)h1;
      const _Float16 h2 = am_f16(r1);
      const _Float16 h3 = am_f16(r1 - (float)h2);
      ra0 = v8h{hi[0], hi[1], hi[2], hi[3], lo[0], lo[1], lo[2], lo[3]};
      ra1 = v8h{h1, h2, h3, one, one, one, zero, zero};
      rn = nn;
    }
  };
  auto commit = [&](int buf) {
    sA[buf][tid >> 5][0][tid & 31] = ra0;
    sA[buf][tid >> 5][1][tid & 31] = ra1;
  };
  auto tiles_of = [&](int ch) { const int left = c - ch * kAmChunk; return left >= kAmChunk ? kAmChunk / 32 : (left + 31) / 32; };
  const v16f zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  // pass 1: min over the centroids of e(c), and the largest |c|^2
  float m[4] = {INFINITY, INFINITY, INFINITY, INFINITY};
  float mycmax = 0.f;
  bool cbad = false;                 // a centroid whose |c|^2 is not a number or not finite
  fetch(0);
  commit(0);
  mycmax = rn;
  cbad = !(rn < INFINITY);
  __syncthreads();
  for (int ch = 0; ch < nchunk; ++ch) {
    const int buf = ch & 1;
    if (ch + 1 < nchunk) fetch(ch + 1);
    const int ntile = tiles_of(ch);
    for (int t = 0; t < ntile; ++t) {
      const v8h a = sA[buf][t][kb][col];
      v16f d[4];
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) d[tt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, bop[tt], zero16, 0, 0, 0);
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) {
        float mm = m[tt];
#pragma unroll
        for (int j = 0; j < 16; j += 2) mm = fminf(fminf(mm, d[tt][j]), d[tt][j + 1]);
        m[tt] = mm;
      }
    }
    if (ch + 1 < nchunk) {
      commit(buf ^ 1);
      cbad = cbad || !(rn < INFINITY);
      if (rn > mycmax) mycmax = rn;
    }
    __syncthreads();
  }
  if (cbad) mycmax = INFINITY;
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) mycmax = fmaxf(mycmax, __shfl_xor(mycmax, o));
  if (lane == 0) s_cmax[w] = mycmax;
  __syncthreads();
  float cmax2 = s_cmax[0];
#pragma unroll
  for (int x = 1; x < 8; ++x) cmax2 = fmaxf(cmax2, s_cmax[x]);

  // thresholds into the B operands of k block 1; tokens out of range take the exact chain over everything
  bool full[4];
#pragma unroll
  for (int tt = 0; tt < 4; ++tt) {
    float mm = fminf(m[tt], __shfl_xor(m[tt], 32));
    const float S = x2[tt] + cmax2;
    full[tt] = !(S < 32768.f) || !(mm == mm) || !(fabsf(mm) < 65000.f);
    const float thr = mm + 2.f * (S * 1.52587890625e-5f + 4.76837158203125e-7f);      // 2^-16 S + 2^-21
    const float tneg = full[tt] ? 0.f : -thr;
    const _Float16 t1 = am_f16(tneg);
    const float r1 = tneg - (float)t1;
    const _Float16 t2 = am_f16(r1);
    const _Float16 t3 = am_f16(r1 - (float)t2);
    if (kb == 1) { bop[tt][3] = t1; bop[tt][4] = t2; bop[tt][5] = t3; }
    if (full[tt]) {
      // no shortlist for this token: x = 0 and t = +1 make every result of pass 2 |c|^2 / 2 + 1 > 0
      const _Float16 one = (_Float16)1.f, zero = (_Float16)0.f;
      if (kb == 0) bop[tt] = v8h{zero, zero, zero, zero, zero, zero, zero, zero};
      else bop[tt] = v8h{one, one, one, one, zero, zero, zero, zero};
    }
  }

  // pass 2: the same products with the threshold folded in; negative results are candidates
  int cand[4][kAmCand];
  int ncand[4] = {0, 0, 0, 0};
  float rest_d[4] = {INFINITY, INFINITY, INFINITY, INFINITY};      // best of the candidates that found the list full
  int rest_i[4] = {0x7fffffff, 0x7fffffff, 0x7fffffff, 0x7fffffff};
#pragma unroll
  for (int tt = 0; tt < 4; ++tt)
#pragma unroll
    for (int q = 0; q < kAmCand; ++q) cand[tt][q] = 0;
  fetch(0);
  commit(0);
  __syncthreads();
  for (int ch = 0; ch < nchunk; ++ch) {
    const int buf = ch & 1;
    if (ch + 1 < nchunk) fetch(ch + 1);
    const int ntile = tiles_of(ch);
    for (int t = 0; t < ntile; ++t) {
      const v8h a = sA[buf][t][kb][col];
      v16f d[4];
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) d[tt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, bop[tt], zero16, 0, 0, 0);
      uint32_t sg[4];
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) {
        uint32_t o = 0;
#pragma unroll
        for (int j = 0; j < 16; j += 2) o = o | __float_as_uint(d[tt][j]) | __float_as_uint(d[tt][j + 1]);
        sg[tt] = o;
      }
      const uint32_t any = sg[0] | sg[1] | sg[2] | sg[3];
      if (__builtin_amdgcn_ballot_w64((int32_t)any < 0) == 0) continue;     // mostly: no candidate in these 32 x 128
      const int cbase = ch * kAmChunk + t * 32 + 4 * kb;
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) {
        if (__builtin_amdgcn_ballot_w64((int32_t)sg[tt] < 0) == 0) continue;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          // rows of the 32x32 result held by this lane: 8 * (j / 4) + 4 * kb + j % 4, ascending in j
          if ((int32_t)__float_as_uint(d[tt][j]) < 0) {
            const int cidx = cbase + 8 * (j >> 2) + (j & 3);
            if (cidx < c) {
#pragma unroll
              for (int q = 0; q < kAmCand; ++q)
                if (ncand[tt] == q) cand[tt][q] = cidx;
              if (ncand[tt] >= kAmCand) {
                // the list is full: this one goes through the exact chain now and only the best of these is kept
                // (they arrive in ascending index order, so a strict comparison keeps the first smallest)
                const int64_t tk = tok0 + 32 * tt + col;
                const uint16_t* src = k_new + ((int64_t)row * T + (tk < T ? tk : T - 1)) * kHeadDim + grp * DBAR;
                float dist = 0.f;
#pragma unroll
                for (int dd = 0; dd < DBAR; ++dd) {
                  const float e = h2f(src[dd]) - cg[(int64_t)cidx * DBAR + dd];
                  dist = fmaf(e, e, dist);
                }
                if (dist < rest_d[tt]) { rest_d[tt] = dist; rest_i[tt] = cidx; }
              }
              ncand[tt] += 1;
            }
          }
        }
      }
    }
    if (ch + 1 < nchunk) commit(buf ^ 1);
    __syncthreads();
  }

  // the exact chain over the candidates (ascending index per lane), or over every centroid
  const int b = row / n_kv_heads;
#pragma unroll
  for (int tt = 0; tt < 4; ++tt) {
    float bd = INFINITY;
    int bi = 0x7fffffff;
    const int64_t t = tok0 + 32 * tt + col;
    float xs[DBAR];
    {
      const uint16_t* src = k_new + ((int64_t)row * T + (t < T ? t : T - 1)) * kHeadDim + grp * DBAR;
#pragma unroll
      for (int dd = 0; dd < DBAR; ++dd) xs[dd] = h2f(src[dd]);
    }
    auto exact = [&](int cidx) {
      float dist = 0.f;
#pragma unroll
      for (int dd = 0; dd < DBAR; ++dd) {
        const float e = xs[dd] - cg[(int64_t)cidx * DBAR + dd];
        dist = fmaf(e, e, dist);
      }
      return dist;
    };
    if (full[tt]) {
      for (int cidx = kb; cidx < c; cidx += 2) {
        const float dist = exact(cidx);
        if (dist < bd) { bd = dist; bi = cidx; }
      }
    } else {
#pragma unroll
      for (int q = 0; q < kAmCand; ++q) {
        if (q < ncand[tt]) {
          const float dist = exact(cand[tt][q]);
          if (dist < bd) { bd = dist; bi = cand[tt][q]; }
        }
      }
      if (rest_d[tt] < bd) { bd = rest_d[tt]; bi = rest_i[tt]; }       // later indices than the list's
    }
    const float od = __shfl_xor(bd, 32);
    const int ob = __shfl_xor(bi, 32);
    if (od < bd || (od == bd && ob < bi)) { bd = od; bi = ob; }
    // the ascending scan starts from centroid 0 whatever its distance: no finite distance at all, or a first
    // distance that is not a number, leave it the winner
    const float d0 = exact(0);
    const int win = (bi == 0x7fffffff || d0 != d0) ? 0 : bi;
    if (kb == 0 && t < T) {
      const int64_t slot = nr.n[b] + t;
      if constexpr (WIDE) reinterpret_cast<uint16_t*>(pcache)[vq_wide_at(g, vq_tiles(cap), row, slot, grp)] = (uint16_t)win;
      else pcache[((int64_t)row * cap + slot) * g + vq_byte_of(grp, slot)] = (uint8_t)win;
      if (grp == 0) {
        if (acc != nullptr) acc[(int64_t)row * cap + slot] = 0.0f;
        if (pos != nullptr) pos[(int64_t)row * cap + slot] = (int32_t)(vrow0.n[b] + t);
      }
    }
  }
}

// Few tokens per call (decode appends): one workgroup per (token, row, four groups); a wave takes one group
// and spreads the group's centroids over its lanes (lane, lane + 64, ...; four distances in flight per lane),
// then the lanes' candidates are reduced by (distance, index): the smaller distance wins, equal distances go
// to the lower index - the same winner as the ascending scan with a strict comparison.
template <int DBAR, bool WIDE>
__global__ __launch_bounds__(256) void vq_assign_small_kernel(int g, int c, int n_kv_heads, int64_t cap,
                                                              const float* __restrict__ centroids,
                                                              uint8_t* __restrict__ pcache,
                                                              const uint16_t* __restrict__ k_new, int64_t T, NRes nr,
                                                              float* __restrict__ acc, int32_t* __restrict__ pos,
                                                              NRes vrow0) {
  const int row = blockIdx.y;
  const int64_t tt = blockIdx.x;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int b = row / n_kv_heads;
  const int64_t slot = nr.n[b] + tt;
  const uint16_t* src = k_new + ((int64_t)row * T + tt) * kHeadDim;
  const float* cb = centroids + (int64_t)(row % n_kv_heads) * g * c * DBAR;
  const int i = blockIdx.z * 4 + w;
  if (i < g) {
    float x[DBAR];
#pragma unroll
    for (int dd = 0; dd < DBAR; ++dd) x[dd] = h2f(src[i * DBAR + dd]);
    float bd = INFINITY;
    int best = 0x7fffffff;
    for (int c0 = lane; c0 < c; c0 += 256) {
      float cv[4][DBAR];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int cc = c0 + 64 * u < c ? c0 + 64 * u : c0;
        const float* p = cb + ((int64_t)i * c + cc) * DBAR;
#pragma unroll
        for (int dd = 0; dd < DBAR; ++dd) cv[u][dd] = p[dd];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int cc = c0 + 64 * u;
        if (cc < c) {
          float d = 0.f;
#pragma unroll
          for (int dd = 0; dd < DBAR; ++dd) {
            const float e = x[dd] - cv[u][dd];
            d = fmaf(e, e, d);
          }
          if (d < bd || best == 0x7fffffff) { bd = d; best = cc; }
        }
      }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      const float od = __shfl_xor(bd, o);
      const int ob = __shfl_xor(best, o);
      if (ob != 0x7fffffff && (best == 0x7fffffff || od < bd || (od == bd && ob < best))) { bd = od; best = ob; }
    }
    if (lane == 0) {
      if constexpr (WIDE) reinterpret_cast<uint16_t*>(pcache)[vq_wide_at(g, vq_tiles(cap), row, slot, i)] = (uint16_t)best;
      else pcache[((int64_t)row * cap + slot) * g + vq_byte_of(i, slot)] = (uint8_t)best;
    }
  }
  if (threadIdx.x == 0 && blockIdx.z == 0) {
    if (acc != nullptr) acc[(int64_t)row * cap + slot] = 0.0f;
    if (pos != nullptr) pos[(int64_t)row * cap + slot] = (int32_t)(vrow0.n[b] + tt);
  }
}

// -------------------------------------------------------------------------------- table ---
// T[row][cc][i][h] (narrow form; T[row][i][cc][h] in the wide form) = qbar_i . C[i][cc] for the G query heads of the row: t = 0; t = fmaf(q, c, t) over
// the group's channels in ascending order.  grid (g, rows), centroids spread over the threads.  The workgroup also
// leaves the largest magnitude of its group's entries, per head, in amax[row][i][4] for the scan.
template <int G, int DBAR>
__global__ __launch_bounds__(256) void vq_lut_kernel(int g, int c, int n_kv_heads, bool wide,
                                                     const float* __restrict__ centroids,
                                                     const uint16_t* __restrict__ q, float* __restrict__ lut,
                                                     float* __restrict__ amax) {
  __shared__ float wmax[4][4];
  const int i = blockIdx.x, row = blockIdx.y;
  float m[G];
#pragma unroll
  for (int h = 0; h < G; ++h) m[h] = 0.f;
  float qv[G][DBAR];
#pragma unroll
  for (int h = 0; h < G; ++h)
#pragma unroll
    for (int dd = 0; dd < DBAR; ++dd) qv[h][dd] = h2f(q[((int64_t)row * G + h) * kHeadDim + i * DBAR + dd]);
  for (int cc = threadIdx.x; cc < c; cc += 256) {
    const float* cv = centroids + (((int64_t)(row % n_kv_heads) * g + i) * c + cc) * DBAR;
    float* out = lut + (wide ? ((int64_t)row * g + i) * c + cc : ((int64_t)row * c + cc) * g + i) * G;
#pragma unroll
    for (int h = 0; h < G; ++h) {
      float t = 0.f;
#pragma unroll
      for (int dd = 0; dd < DBAR; ++dd) t = fmaf(qv[h][dd], cv[dd], t);
      out[h] = t;
      m[h] = fmaxf(m[h], fabsf(t));
    }
  }
#pragma unroll
  for (int h = 0; h < G; ++h) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m[h] = fmaxf(m[h], __shfl_xor(m[h], o));
    if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6][h] = m[h];
  }
  __syncthreads();
  if (threadIdx.x < G)
    amax[((int64_t)row * g + i) * 4 + threadIdx.x] = fmaxf(fmaxf(wmax[0][threadIdx.x], wmax[1][threadIdx.x]),
                                                           fmaxf(wmax[2][threadIdx.x], wmax[3][threadIdx.x]));
}

// --------------------------------------------------------------------------------- scan ---
template <int G> struct EntryT;
template <> struct EntryT<4> { using type = float4; using fix = int4; };
template <> struct EntryT<2> { using type = float2; using fix = int2; };
template <> struct EntryT<1> { using type = float; using fix = int; };

template <int G>
__device__ __forceinline__ void entry_absmax(float (&m)[G], const typename EntryT<G>::type& e) {
  if constexpr (G == 4) {
    m[0] = fmaxf(m[0], fabsf(e.x)); m[1] = fmaxf(m[1], fabsf(e.y));
    m[2] = fmaxf(m[2], fabsf(e.z)); m[3] = fmaxf(m[3], fabsf(e.w));
  } else if constexpr (G == 2) {
    m[0] = fmaxf(m[0], fabsf(e.x)); m[1] = fmaxf(m[1], fabsf(e.y));
  } else {
    m[0] = fmaxf(m[0], fabsf(e));
  }
}
template <int G>
__device__ __forceinline__ typename EntryT<G>::fix entry_fix(const typename EntryT<G>::type& e, const int* s) {
  typename EntryT<G>::fix r;
  if constexpr (G == 4) {
    r.x = vq_fix(e.x, s[0]); r.y = vq_fix(e.y, s[1]); r.z = vq_fix(e.z, s[2]); r.w = vq_fix(e.w, s[3]);
  } else if constexpr (G == 2) {
    r.x = vq_fix(e.x, s[0]); r.y = vq_fix(e.y, s[1]);
  } else {
    r = vq_fix(e, s[0]);
  }
  return r;
}
template <int G>
__device__ __forceinline__ void entry_add2(int (&z)[G], const typename EntryT<G>::fix& a,
                                           const typename EntryT<G>::fix& b) {
  if constexpr (G == 4) {
    z[0] = z[0] + a.x + b.x; z[1] = z[1] + a.y + b.y; z[2] = z[2] + a.z + b.z; z[3] = z[3] + a.w + b.w;
  } else if constexpr (G == 2) {
    z[0] = z[0] + a.x + b.x; z[1] = z[1] + a.y + b.y;
  } else {
    z[0] = z[0] + a + b;
  }
}

// Eq. 3.  One workgroup of 1024 threads reduces the per-group maxima to the largest magnitude of each
// query head's table and copies the row's table (c * g entries of G floats) into LDS on that head's
// power-of-two grid (24 bits for the largest entry, vq_fix).  Then each thread scores one
// token at a time: NG index bytes (two or four 16-byte loads; a wave reads 64 consecutive tokens = 2 or
// 4 KiB in one piece, the next token's bytes are on their way while this one's are looked up), NG table
// reads, an exact integer sum - so the order of the additions is free and two entries go into one
// three-operand add - and one conversion back to fp32.  With the largest supported table (128 KiB) one
// workgroup fits a compute unit, so the launch has about one workgroup per unit and each takes an
// equal share of the row.  Shares start at multiples of 1024 slots: a thread's tokens all have its own
// lane number modulo 16, which makes the rotation of the index bytes a per-thread constant.
template <int G, int NG>
__global__ __launch_bounds__(1024) void vq_scan_kernel(int c, int64_t cap, const uint8_t* __restrict__ pcache,
                                                       float* __restrict__ lut, NRes nr, int n_kv_heads,
                                                       int64_t per_wg, float* __restrict__ sel, float* __restrict__ z_out) {
  using E = typename EntryT<G>::type;
  using F = typename EntryT<G>::fix;
  constexpr int ES = 4 * G;                              // bytes per table entry
  constexpr int kAhead = 1;                              // tokens whose index bytes are in flight per thread (deeper: slower)
  extern __shared__ __align__(16) unsigned char lds_raw[];
  __shared__ int sexp[4];
  const int row = blockIdx.y;
  const int64_t n = nr.n[row / n_kv_heads];
  const int64_t j0 = (int64_t)blockIdx.x * per_wg;
  if (j0 >= n) return;
  int64_t j1 = j0 + per_wg;
  if (j1 > n) j1 = n;
  const uint8_t* prow = pcache + (int64_t)row * cap * NG;
  int64_t j = j0 + threadIdx.x;
  uint4 nx[kAhead][NG / 16];                             // the index bytes of this thread's next kAhead tokens
#pragma unroll
  for (int d = 0; d < kAhead; ++d)
    if (j + 1024 * d < j1) {
#pragma unroll
      for (int v = 0; v < NG / 16; ++v) nx[d][v] = reinterpret_cast<const uint4*>(prow + (j + 1024 * d) * NG)[v];
    }
  {
    // exponents of the heads' grids from the per-group maxima the table kernel left behind the table
    float* tail = lut + (int64_t)gridDim.y * NG * c * G;
    if (threadIdx.x < 64) {
      const float* am = tail + (int64_t)row * NG * 4;
      const int h = threadIdx.x & 3, part = threadIdx.x >> 2;          // 16 lanes per head
      float m = 0.f;
      if (h < G)
        for (int i = part; i < NG; i += 16) m = fmaxf(m, am[i * 4 + h]);
#pragma unroll
      for (int o = 32; o >= 4; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
      if (threadIdx.x < G) {
        const int s = vq_grid_exponent(m);
        sexp[threadIdx.x] = s;
        if (blockIdx.x == 0)                             // kept for the attend kernels
          reinterpret_cast<int32_t*>(tail + (int64_t)gridDim.y * NG * 4)[row * 4 + threadIdx.x] = s;
      }
    }
    __syncthreads();
    int s[G];
#pragma unroll
    for (int h = 0; h < G; ++h) s[h] = sexp[h];
    const E* src = reinterpret_cast<const E*>(lut) + (int64_t)row * NG * c;
    F* tabi = reinterpret_cast<F*>(lds_raw);
    for (int i = threadIdx.x; i < NG * c; i += 1024) tabi[i] = entry_fix<G>(src[i], s);
    __syncthreads();
  }
  int sx[G];
#pragma unroll
  for (int h = 0; h < G; ++h) sx[h] = -sexp[h];
  const uint32_t l16 = threadIdx.x & 15u;
  uint32_t off[16];
#pragma unroll
  for (int b = 0; b < 16; ++b) off[b] = ((b + l16) & 15u) * ES;
  for (; j < j1; j += 1024 * kAhead) {
#pragma unroll
    for (int d = 0; d < kAhead; ++d) {
      const int64_t jj = j + 1024 * d;
      if (jj >= j1) break;
      uint4 pw[NG / 16];
#pragma unroll
      for (int v = 0; v < NG / 16; ++v) pw[v] = nx[d][v];
      if (jj + 1024 * kAhead < j1) {
#pragma unroll
        for (int v = 0; v < NG / 16; ++v)
          nx[d][v] = reinterpret_cast<const uint4*>(prow + (jj + 1024 * kAhead) * NG)[v];
      }
      int zi[G];
#pragma unroll
      for (int h = 0; h < G; ++h) zi[h] = 0;
#pragma unroll
      for (int v = 0; v < NG / 16; ++v) {
        const uint32_t wd[4] = {pw[v].x, pw[v].y, pw[v].z, pw[v].w};
        F e[16];                                         // sixteen table reads in flight
#pragma unroll
        for (int b = 0; b < 16; ++b) {
          const uint32_t code = (wd[b >> 2] >> (8 * (b & 3))) & 255u;
          e[b] = *reinterpret_cast<const F*>(lds_raw + code * (NG * ES) + off[b] + 16 * v * ES);
        }
#pragma unroll
        for (int b = 0; b < 16; b += 2) entry_add2<G>(zi, e[b], e[b + 1]);
      }
      float z[G];
#pragma unroll
      for (int h = 0; h < G; ++h) z[h] = ldexpf((float)zi[h], sx[h]);
      float best = z[0];
#pragma unroll
      for (int h = 1; h < G; ++h) best = fmaxf(best, z[h]);
      sel[(int64_t)row * cap + jj] = best;
      if (z_out != nullptr) {
#pragma unroll
        for (int h = 0; h < G; ++h) z_out[((int64_t)row * G + h) * cap + jj] = z[h];
      }
    }
  }
}

// Eq. 3 for the wide form (16-bit indices, a table larger than LDS).  One workgroup of 1024 threads scans
// one tile of 16 Ki slots, 16 consecutive slots per thread with their running integer sums in registers,
// and walks through the groups a slice at a time: gps groups whose entries (gps * c * G * 4 bytes <= 128 KiB)
// are copied from the group-major table into LDS on their heads' grids, then looked up with the tile's
// indices of those groups (32 contiguous bytes per thread and group).  The table is re-read once per tile:
// 4 MiB of full lines from L2 per 16 Ki tokens, instead of one L2 request per token and group.
template <int G>
__global__ __launch_bounds__(1024) void vq_scan_wide_kernel(int g, int c, int gps, int64_t cap,
                                                             const uint16_t* __restrict__ pcache,
                                                             float* __restrict__ lut, NRes nr, int n_kv_heads, int rows,
                                                             float* __restrict__ sel, float* __restrict__ z_out) {
  using E = typename EntryT<G>::type;
  using F = typename EntryT<G>::fix;
  extern __shared__ __align__(16) unsigned char lds_raw[];
  __shared__ int sexp[4];
  // workgroup x serves row x % rows: consecutive workgroups go to the eight dies in turn, so with eight rows
  // every row is scanned by one die and its table (4 MiB at c = 8192, four query heads) stays in that die's L2
  const int row = blockIdx.x % rows;
  const int64_t tile = blockIdx.x / rows;
  const int64_t n = nr.n[row / n_kv_heads];
  const int64_t t0 = tile * kVqTile;
  if (t0 >= n) return;
  float* tail = lut + (int64_t)rows * g * c * G;
  if (threadIdx.x < 64) {                                 // exponents from the per-group maxima, as in the LDS form
    const float* am = tail + (int64_t)row * g * 4;
    const int h = threadIdx.x & 3, part = threadIdx.x >> 2;
    float m = 0.f;
    if (h < G)
      for (int i = part; i < g; i += 16) m = fmaxf(m, am[i * 4 + h]);
#pragma unroll
    for (int o = 32; o >= 4; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if (threadIdx.x < G) {
      const int s = vq_grid_exponent(m);
      sexp[threadIdx.x] = s;
      if (tile == 0) reinterpret_cast<int32_t*>(tail + (int64_t)rows * g * 4)[row * 4 + threadIdx.x] = s;
    }
  }
  __syncthreads();
  int s[G];
#pragma unroll
  for (int h = 0; h < G; ++h) s[h] = sexp[h];
  F* tab = reinterpret_cast<F*>(lds_raw);
  const E* trow = reinterpret_cast<const E*>(lut) + (int64_t)row * g * c;
  const int64_t tiles = vq_tiles(cap);
  const uint16_t* ptile = pcache + (row * tiles + tile) * g * (int64_t)kVqTile + threadIdx.x * 16;
  int zi[16][G];
#pragma unroll
  for (int tt = 0; tt < 16; ++tt)
#pragma unroll
    for (int h = 0; h < G; ++h) zi[tt][h] = 0;
  // the indices of the next group are fetched while the current group is looked up (and while the next slice
  // of the table is brought in), so no slice waits for HBM
  auto load_idx = [](const uint16_t* p, int i) {          // read once: keep it out of the way of the table in L2
    const v4i t4 = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(p) + i);
    return uint4{(uint32_t)t4.x, (uint32_t)t4.y, (uint32_t)t4.z, (uint32_t)t4.w};
  };
  uint4 na = load_idx(ptile, 0), nb = load_idx(ptile, 1);
  for (int g0 = 0; g0 < g; g0 += gps) {
    __syncthreads();                                      // the previous slice's lookups are done
    const E* src = trow + (int64_t)g0 * c;
    for (int i = threadIdx.x; i < gps * c; i += 1024) tab[i] = entry_fix<G>(src[i], s);
    __syncthreads();
    for (int gl = 0; gl < gps; ++gl) {
      const uint4 pa = na, pb = nb;
      if (g0 + gl + 1 < g) {
        const uint16_t* ip = ptile + (int64_t)(g0 + gl + 1) * kVqTile;
        na = load_idx(ip, 0);
        nb = load_idx(ip, 1);
      }
      const uint32_t wd[8] = {pa.x, pa.y, pa.z, pa.w, pb.x, pb.y, pb.z, pb.w};
      F e[16];                                            // sixteen table reads in flight
#pragma unroll
      for (int tt = 0; tt < 16; ++tt) {
        uint32_t code = (wd[tt >> 1] >> (16 * (tt & 1))) & 0xffffu;
        if (code >= (uint32_t)c) code = 0;                // slots past n hold whatever memory held
        e[tt] = tab[gl * c + code];
      }
#pragma unroll
      for (int tt = 0; tt < 16; ++tt) {
        if constexpr (G == 4) { zi[tt][0] += e[tt].x; zi[tt][1] += e[tt].y; zi[tt][2] += e[tt].z; zi[tt][3] += e[tt].w; }
        else if constexpr (G == 2) { zi[tt][0] += e[tt].x; zi[tt][1] += e[tt].y; }
        else { zi[tt][0] += e[tt]; }
      }
    }
  }
  const int64_t j0 = t0 + threadIdx.x * 16;
#pragma unroll
  for (int tt = 0; tt < 16; ++tt) {
    const int64_t j = j0 + tt;
    if (j >= n) break;
    float z[G];
#pragma unroll
    for (int h = 0; h < G; ++h) z[h] = ldexpf((float)zi[tt][h], -s[h]);
    float best = z[0];
#pragma unroll
    for (int h = 1; h < G; ++h) best = fmaxf(best, z[h]);
    sel[(int64_t)row * cap + j] = best;
    if (z_out != nullptr) {
#pragma unroll
      for (int h = 0; h < G; ++h) z_out[((int64_t)row * G + h) * cap + j] = z[h];
    }
  }
}

// Canonical export of the index rows for tests: out[row][slot][group], slots < n_resident.
__global__ __launch_bounds__(256) void vq_export_kernel(int g, int64_t cap, const uint8_t* __restrict__ pcache, NRes nr,
                                                        int n_kv_heads, uint8_t* __restrict__ out) {
  const int row = blockIdx.y;
  const int64_t n = nr.n[row / n_kv_heads];
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t slot = gid / g;
  const int i = (int)(gid % g);
  if (slot >= n) return;
  out[((int64_t)row * cap + slot) * g + i] = pcache[((int64_t)row * cap + slot) * g + vq_byte_of(i, slot)];
}

__global__ __launch_bounds__(256) void vq_export_wide_kernel(int g, int64_t cap, const uint16_t* __restrict__ pcache,
                                                             NRes nr, int n_kv_heads, uint16_t* __restrict__ out) {
  const int row = blockIdx.y;
  const int64_t n = nr.n[row / n_kv_heads];
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (gid >= n * g) return;
  const int64_t slot = gid / g;
  const int i = (int)(gid % g);
  out[(int64_t)row * cap * g + gid] = pcache[vq_wide_at(g, vq_tiles(cap), row, slot, i)];
}

int32_t launch_vq_assign(const Layout& L, int g, int c, const float* centroids, uint8_t* pcache, const void* k_new,
                         int64_t T, const NRes& nr, float* acc_opt, int32_t* pos_opt, const NRes& vrow0, hipStream_t st) {
  if (T == 0) return HCA_OK;
  const uint16_t* kn = (const uint16_t*)k_new;
  const bool wide = vq_is_wide(L, g, c);
#define HCA_ASSIGN(KERNEL, GRID)                                                                                      \
  do {                                                                                                                \
    if (g == 32 && wide) KERNEL<4, true><<<GRID, 256, 0, st>>>(g, c, L.n_kv_heads, L.cap, centroids, pcache, kn, T, nr, acc_opt, pos_opt, vrow0); \
    else if (g == 32) KERNEL<4, false><<<GRID, 256, 0, st>>>(g, c, L.n_kv_heads, L.cap, centroids, pcache, kn, T, nr, acc_opt, pos_opt, vrow0);   \
    else if (wide) KERNEL<2, true><<<GRID, 256, 0, st>>>(g, c, L.n_kv_heads, L.cap, centroids, pcache, kn, T, nr, acc_opt, pos_opt, vrow0);      \
    else KERNEL<2, false><<<GRID, 256, 0, st>>>(g, c, L.n_kv_heads, L.cap, centroids, pcache, kn, T, nr, acc_opt, pos_opt, vrow0);               \
  } while (0)
#define HCA_ASSIGN_B(GPW, GRID)                                                                                       \
  do {                                                                                                                \
    if (g == 32 && wide) vq_assign_kernel<4, true, GPW><<<GRID, 256, 0, st>>>(g, c, L.n_kv_heads, L.cap, centroids, pcache, kn, T, nr, acc_opt, pos_opt, vrow0); \
    else if (g == 32) vq_assign_kernel<4, false, GPW><<<GRID, 256, 0, st>>>(g, c, L.n_kv_heads, L.cap, centroids, pcache, kn, T, nr, acc_opt, pos_opt, vrow0);   \
    else if (wide) vq_assign_kernel<2, true, GPW><<<GRID, 256, 0, st>>>(g, c, L.n_kv_heads, L.cap, centroids, pcache, kn, T, nr, acc_opt, pos_opt, vrow0);      \
    else vq_assign_kernel<2, false, GPW><<<GRID, 256, 0, st>>>(g, c, L.n_kv_heads, L.cap, centroids, pcache, kn, T, nr, acc_opt, pos_opt, vrow0);               \
  } while (0)
  if (T >= kAssignMfmaMinTokens && c >= kAssignMfmaMinCodewords && T * c >= kAssignMfmaMinWork) {
    // a block or a context: shortlist on the matrix cores, exact chain on the shortlist
    dim3 gm((unsigned)((T + 1023) / 1024), (unsigned)L.rows, (unsigned)g);
    if (g == 32 && wide) vq_assign_mfma_kernel<4, true><<<gm, 512, 0, st>>>(g, c, L.n_kv_heads, L.cap, centroids, pcache, kn, T, nr, acc_opt, pos_opt, vrow0);
    else if (g == 32) vq_assign_mfma_kernel<4, false><<<gm, 512, 0, st>>>(g, c, L.n_kv_heads, L.cap, centroids, pcache, kn, T, nr, acc_opt, pos_opt, vrow0);
    else if (wide) vq_assign_mfma_kernel<2, true><<<gm, 512, 0, st>>>(g, c, L.n_kv_heads, L.cap, centroids, pcache, kn, T, nr, acc_opt, pos_opt, vrow0);
    else vq_assign_mfma_kernel<2, false><<<gm, 512, 0, st>>>(g, c, L.n_kv_heads, L.cap, centroids, pcache, kn, T, nr, acc_opt, pos_opt, vrow0);
  } else if (T <= 8) {                              // decode appends: parallel over centroids, not over tokens
    dim3 gs((unsigned)T, (unsigned)L.rows, (unsigned)(g / 4));
    HCA_ASSIGN(vq_assign_small_kernel, gs);
  } else if ((T + 63) / 64 * L.rows * (g / 4) < 16 * 1024) {
    // a block of a few thousand tokens: with four groups per wave the launch would have at most a few waves per
    // SIMD (the chip has 1024 of them); one group per wave gives four times as many
    dim3 grid((unsigned)((T + 63) / 64), (unsigned)L.rows, (unsigned)(g / 4));
    HCA_ASSIGN_B(1, grid);
  } else {
    dim3 grid((unsigned)((T + 63) / 64), (unsigned)L.rows, (unsigned)(g / 16));
    HCA_ASSIGN_B(4, grid);
  }
#undef HCA_ASSIGN_B
#undef HCA_ASSIGN
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

template <int G>
static int32_t scan_wide_launch(const Layout& L, int g, int c, const uint8_t* pcache, float* lut, const NRes& nr,
                                int64_t nmax, float* sel, float* z_opt, hipStream_t st) {
  int gps = 1;                                      // groups per LDS slice: the most that fit 128 KiB
  while (gps * 2 <= g && (int64_t)gps * 2 * c * G * 4 <= 128 * 1024) gps *= 2;
  const size_t lds = (size_t)gps * c * G * 4;
  if (lds > 64 * 1024) {
    static std::atomic<uint64_t> opted{0};                  // one per instantiation
    const int32_t rc = lds_opt_in(reinterpret_cast<const void*>(&vq_scan_wide_kernel<G>), 128 * 1024, &opted);   // + 16 B static
    if (rc != HCA_OK) return rc;
  }
  vq_scan_wide_kernel<G><<<(unsigned)(vq_tiles(nmax) * L.rows), 1024, lds, st>>>(g, c, gps, L.cap, (const uint16_t*)pcache,
                                                                                 lut, nr, L.n_kv_heads, L.rows, sel, z_opt);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

template <int G, int NG>
static int32_t scan_launch(const Layout& L, int c, const uint8_t* pcache, float* lut, const NRes& nr,
                           int64_t nmax, float* sel, float* z_opt, hipStream_t st) {
  const size_t lds = (size_t)NG * c * G * 4;
  if (lds > 64 * 1024) {                            // tables beyond 64 KiB need the opt-in, once per device
    static std::atomic<uint64_t> opted{0};          // one per instantiation
    const int32_t rc = lds_opt_in(reinterpret_cast<const void*>(&vq_scan_kernel<G, NG>), 128 * 1024, &opted);   // + 272 B static
    if (rc != HCA_OK) return rc;
  }
  // about one workgroup per compute unit, each with at least 1024 tokens, shares a multiple of 1024
  int64_t per_row = 256 / L.rows;
  if (per_row < 1) per_row = 1;
  int64_t per_wg = align_up((nmax + per_row - 1) / per_row, 1024);
  const int64_t chunks = (nmax + per_wg - 1) / per_wg;
  dim3 grid((unsigned)chunks, (unsigned)L.rows);
  vq_scan_kernel<G, NG><<<grid, 1024, lds, st>>>(c, L.cap, pcache, lut, nr, L.n_kv_heads, per_wg, sel, z_opt);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

int32_t launch_vq_score(const Layout& L, int g, int c, const float* centroids, const uint8_t* pcache, const void* q,
                        const NRes& nr, int64_t nmax, float* lut, float* sel, float* z_opt, hipStream_t st) {
  const uint16_t* qq = (const uint16_t*)q;
  dim3 gl((unsigned)g, (unsigned)L.rows);
  float* amax = lut + (int64_t)L.rows * g * c * L.gqa;   // [rows][g][4], then the exponents [rows][4]
#define HCA_LUT(G, D) vq_lut_kernel<G, D><<<gl, 256, 0, st>>>(g, c, L.n_kv_heads, vq_is_wide(L, g, c), centroids, qq, lut, amax)
  if (g == 32) {
    if (L.gqa == 4) HCA_LUT(4, 4); else if (L.gqa == 2) HCA_LUT(2, 4); else HCA_LUT(1, 4);
  } else {
    if (L.gqa == 4) HCA_LUT(4, 2); else if (L.gqa == 2) HCA_LUT(2, 2); else HCA_LUT(1, 2);
  }
#undef HCA_LUT
  HCA_HIP(hipGetLastError());
  if (nmax == 0) return HCA_OK;
  if (vq_is_wide(L, g, c)) {
    if (L.gqa == 4) return scan_wide_launch<4>(L, g, c, pcache, lut, nr, nmax, sel, z_opt, st);
    if (L.gqa == 2) return scan_wide_launch<2>(L, g, c, pcache, lut, nr, nmax, sel, z_opt, st);
    return scan_wide_launch<1>(L, g, c, pcache, lut, nr, nmax, sel, z_opt, st);
  }
  if (g == 32) {
    if (L.gqa == 4) return scan_launch<4, 32>(L, c, pcache, lut, nr, nmax, sel, z_opt, st);
    if (L.gqa == 2) return scan_launch<2, 32>(L, c, pcache, lut, nr, nmax, sel, z_opt, st);
    return scan_launch<1, 32>(L, c, pcache, lut, nr, nmax, sel, z_opt, st);
  }
  if (L.gqa == 4) return scan_launch<4, 64>(L, c, pcache, lut, nr, nmax, sel, z_opt, st);
  if (L.gqa == 2) return scan_launch<2, 64>(L, c, pcache, lut, nr, nmax, sel, z_opt, st);
  return scan_launch<1, 64>(L, c, pcache, lut, nr, nmax, sel, z_opt, st);
}

// Shape checks shared by the entry points: the uniform-code fields of the shape are not used here.
static int32_t vq_layout(const hca_shape* shape, const hca_vq_codebook* cb, Layout* L, bool need_centroids) {
  if (shape == nullptr || cb == nullptr) return HCA_ERR_BAD_ARG;
  hca_shape s = *shape;
  s.bits = 4;
  s.group = 32;
  int32_t rc = make_layout(&s, L);
  if (rc != HCA_OK) return rc;
  if (cb->groups != 32 && cb->groups != 64) return HCA_ERR_UNSUPPORTED;
  if (cb->codewords < 1) return HCA_ERR_BAD_ARG;
  if (cb->codewords > 8192) return HCA_ERR_UNSUPPORTED;
  if (need_centroids && cb->centroids == nullptr) return HCA_ERR_BAD_ARG;
  return HCA_OK;
}

// ------------------------------------------------------------------------------ trainer ---
// Lloyd's k-means, one codebook per group (or one for the pooled sub-vectors), codebooks spread over
// host threads.  Within a codebook everything runs in pool order, so the result does not depend on
// the number of threads.
static void train_one(const uint16_t* kval, int64_t nval, int D, int g, int c, int dbar, bool shared, int b,
                      const int32_t* init, int iters, float* cb, double* iner, std::atomic<int>* bad) {
  const int64_t npool = shared ? nval * g : nval;
  std::vector<float> x((size_t)npool * dbar);
  auto half = [](uint16_t h) -> float {
    _Float16 v;
    std::memcpy(&v, &h, 2);
    return (float)v;
  };
  for (int64_t p = 0; p < npool; ++p) {
    const int64_t t = shared ? p / g : p;
    const int i = shared ? (int)(p % g) : b;
    for (int dd = 0; dd < dbar; ++dd) x[(size_t)p * dbar + dd] = half(kval[t * D + i * dbar + dd]);
  }
  for (int cc = 0; cc < c; ++cc) {
    int64_t s = init[cc];
    if (s < 0 || s >= npool) { bad->store(1); s = 0; }
    std::memcpy(cb + (size_t)cc * dbar, &x[(size_t)s * dbar], sizeof(float) * dbar);
  }
  std::vector<double> sum((size_t)c * dbar);
  std::vector<int64_t> cnt((size_t)c);
  for (int it = 0; it <= iters; ++it) {
    std::fill(sum.begin(), sum.end(), 0.0);
    std::fill(cnt.begin(), cnt.end(), (int64_t)0);
    double obj = 0.0;
    for (int64_t p = 0; p < npool; ++p) {
      const float* xp = &x[(size_t)p * dbar];
      int best = 0;
      float bd = 0.f;
      for (int cc = 0; cc < c; ++cc) {
        const float* cv = cb + (size_t)cc * dbar;
        float d = 0.f;
        for (int dd = 0; dd < dbar; ++dd) {
          const float e = xp[dd] - cv[dd];
          d = std::fmaf(e, e, d);
        }
        if (cc == 0 || d < bd) { bd = d; best = cc; }
      }
      obj += (double)bd;
      cnt[best] += 1;
      for (int dd = 0; dd < dbar; ++dd) sum[(size_t)best * dbar + dd] += (double)xp[dd];
    }
    iner[it] = obj;
    if (it == iters) break;
    for (int cc = 0; cc < c; ++cc)
      if (cnt[cc] > 0)
        for (int dd = 0; dd < dbar; ++dd) cb[(size_t)cc * dbar + dd] = (float)(sum[(size_t)cc * dbar + dd] / (double)cnt[cc]);
  }
}

}  // namespace hca

using namespace hca;

extern "C" {

size_t hca_vq_pcache_bytes(const hca_shape* shape, const hca_vq_codebook* cb) {
  Layout L;
  if (vq_layout(shape, cb, &L, false) != HCA_OK) return 0;
  if (vq_is_wide(L, cb->groups, cb->codewords))      // whole tiles of 16 Ki slots
    return (size_t)L.rows * (size_t)vq_tiles(L.cap) * kVqTile * (size_t)cb->groups * 2;
  return (size_t)L.rows * (size_t)L.cap * (size_t)cb->groups;
}

size_t hca_vq_workspace_bytes(const hca_shape* shape, const hca_vq_codebook* cb, int64_t k_max, int64_t m_max) {
  Layout L;
  if (vq_layout(shape, cb, &L, false) != HCA_OK) return 0;
  hca_shape s = *shape;      // the hca_vq_* calls lay the workspace out as the 4-bit uniform path does
  s.bits = 4;
  s.group = 32;
  return hca_workspace_bytes(&s, k_max, m_max);
}

size_t hca_vq_lut_bytes(const hca_shape* shape, const hca_vq_codebook* cb) {
  Layout L;
  if (vq_layout(shape, cb, &L, false) != HCA_OK) return 0;
  return (size_t)L.rows * cb->groups * cb->codewords * L.gqa * 4 + (size_t)L.rows * (cb->groups + 1) * 4 * sizeof(int32_t);
}

int32_t hca_vq_train(const void* kval_f16, int64_t n_val, int32_t head_dim, int32_t groups, int32_t codewords,
                     const int32_t* init, int32_t iters, int32_t shared, float* centroids, double* inertia_opt) {
  if (kval_f16 == nullptr || init == nullptr || centroids == nullptr) return HCA_ERR_BAD_ARG;
  if (head_dim < 1 || groups < 1 || head_dim % groups != 0 || codewords < 1 || n_val < 1 || iters < 0)
    return HCA_ERR_BAD_ARG;
  const int dbar = head_dim / groups;
  const int ncb = shared ? 1 : groups;
  std::vector<double> iner((size_t)ncb * (iters + 1), 0.0);
  std::atomic<int> bad{0};
  std::atomic<int> next{0};
  auto work = [&]() {
    for (int b = next.fetch_add(1); b < ncb; b = next.fetch_add(1))
      train_one((const uint16_t*)kval_f16, n_val, head_dim, groups, codewords, dbar, shared != 0, b,
                init + (size_t)b * codewords, iters, centroids + (size_t)b * codewords * dbar,
                &iner[(size_t)b * (iters + 1)], &bad);
  };
  unsigned nt = std::thread::hardware_concurrency();
  if (nt < 1) nt = 1;
  if (nt > 16) nt = 16;
  if ((int)nt > ncb) nt = (unsigned)ncb;
  std::vector<std::thread> pool;
  for (unsigned t = 1; t < nt; ++t) pool.emplace_back(work);
  work();
  for (auto& th : pool) th.join();
  if (shared)
    for (int i = 1; i < groups; ++i)
      std::memcpy(centroids + (size_t)i * codewords * dbar, centroids, sizeof(float) * (size_t)codewords * dbar);
  if (inertia_opt != nullptr)
    for (int it = 0; it <= iters; ++it) {
      double s = 0.0;
      for (int b = 0; b < ncb; ++b) s += iner[(size_t)b * (iters + 1) + it];
      inertia_opt[it] = s;
    }
  return bad.load() ? HCA_ERR_BAD_ARG : HCA_OK;
}

int32_t hca_vq_assign(const hca_shape* shape, const hca_vq_codebook* cb, void* pcache, const void* k_new_f16,
                      int64_t T, const int64_t* n_resident, float* acc_opt, int32_t* pos_opt,
                      const int64_t* value_row0, void* stream) {
  Layout L;
  int32_t rc = vq_layout(shape, cb, &L, true);
  if (rc != HCA_OK) return rc;
  if (pcache == nullptr || T < 0 || (T > 0 && k_new_f16 == nullptr)) return HCA_ERR_BAD_ARG;
  NRes nr, vrow0;
  int64_t nmax;
  rc = load_nres(L, n_resident, &nr, &nmax);
  if (rc != HCA_OK) return rc;
  for (int b = 0; b < L.batch; ++b)
    if (nr.n[b] + T > L.cap) return HCA_ERR_CAPACITY;
  for (int b = 0; b < kMaxBatch; ++b) vrow0.n[b] = 0;
  for (int b = 0; b < L.batch; ++b) vrow0.n[b] = value_row0 ? value_row0[b] : nr.n[b];
  return launch_vq_assign(L, cb->groups, cb->codewords, cb->centroids, (uint8_t*)pcache, k_new_f16, T, nr, acc_opt,
                          pos_opt, vrow0, (hipStream_t)stream);
}

int32_t hca_vq_score(const hca_shape* shape, const hca_vq_codebook* cb, const void* pcache, const void* q_f16,
                     const int64_t* n_resident, float* lut, float* sel, float* z_opt, void* stream) {
  Layout L;
  int32_t rc = vq_layout(shape, cb, &L, true);
  if (rc != HCA_OK) return rc;
  if (pcache == nullptr || q_f16 == nullptr || lut == nullptr || sel == nullptr) return HCA_ERR_BAD_ARG;
  NRes nr;
  int64_t nmax;
  rc = load_nres(L, n_resident, &nr, &nmax);
  if (rc != HCA_OK) return rc;
  return launch_vq_score(L, cb->groups, cb->codewords, cb->centroids, (const uint8_t*)pcache, q_f16, nr, nmax, lut,
                         sel, z_opt, (hipStream_t)stream);
}

int32_t hca_vq_export_pcache(const hca_shape* shape, const hca_vq_codebook* cb, const void* pcache,
                             const int64_t* n_resident, void* indices, void* stream) {
  Layout L;
  int32_t rc = vq_layout(shape, cb, &L, false);
  if (rc != HCA_OK) return rc;
  if (pcache == nullptr || indices == nullptr) return HCA_ERR_BAD_ARG;
  NRes nr;
  int64_t nmax;
  rc = load_nres(L, n_resident, &nr, &nmax);
  if (rc != HCA_OK) return rc;
  if (nmax == 0) return HCA_OK;
  dim3 grid((unsigned)((nmax * cb->groups + 255) / 256), (unsigned)L.rows);
  if (vq_is_wide(L, cb->groups, cb->codewords))
    vq_export_wide_kernel<<<grid, 256, 0, (hipStream_t)stream>>>(cb->groups, L.cap, (const uint16_t*)pcache, nr,
                                                                 L.n_kv_heads, (uint16_t*)indices);
  else
    vq_export_kernel<<<grid, 256, 0, (hipStream_t)stream>>>(cb->groups, L.cap, (const uint8_t*)pcache, nr, L.n_kv_heads,
                                                            (uint8_t*)indices);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

int32_t hca_vq_attend_gathered(const hca_shape* shape, const hca_vq_codebook* cb, const void* pcache,
                               const float* lut, const int32_t* idx, const int32_t* count, int32_t k,
                               float sm_scale, float* y, float* acc_opt, void* workspace, void* stream) {
  Layout L;
  int32_t rc = vq_layout(shape, cb, &L, false);
  if (rc != HCA_OK) return rc;
  if (pcache == nullptr || lut == nullptr || idx == nullptr || count == nullptr || y == nullptr ||
      workspace == nullptr)
    return HCA_ERR_BAD_ARG;
  if (k < 1 || k > L.cap || k > 64 * 256) return HCA_ERR_CAPACITY;
  return launch_vq_attend_gathered(L, cb->groups, cb->codewords, (const uint8_t*)pcache, lut, idx, count, k, sm_scale,
                                   y, acc_opt, workspace, (hipStream_t)stream);
}

int32_t hca_vq_evict(const hca_shape* shape, const hca_vq_codebook* cb, void* pcache, float* acc, int32_t* pos,
                     const int64_t* n_resident, int64_t M, int64_t n_protect, int32_t* kept_opt, void* workspace,
                     void* pcache_dst, float* acc_dst, int32_t* pos_dst, void* stream) {
  Layout L;
  int32_t rc = vq_layout(shape, cb, &L, false);
  if (rc != HCA_OK) return rc;
  if (pcache == nullptr || acc == nullptr || pos == nullptr || workspace == nullptr) return HCA_ERR_BAD_ARG;
  const bool oop = pcache_dst != nullptr || acc_dst != nullptr || pos_dst != nullptr;
  if (oop && (pcache_dst == nullptr || acc_dst == nullptr || pos_dst == nullptr)) return HCA_ERR_BAD_ARG;
  if (oop && (pcache_dst == pcache || acc_dst == acc || pos_dst == pos)) return HCA_ERR_BAD_ARG;
  if (M < 1 || M > L.cap || n_protect < 0 || n_protect > M) return HCA_ERR_CAPACITY;
  NRes nr;
  int64_t nmax;
  rc = load_nres(L, n_resident, &nr, &nmax);
  if (rc != HCA_OK) return rc;
  return launch_vq_evict(L, cb->groups, cb->codewords, (uint8_t*)pcache, acc, pos, nr, nmax, M, n_protect, kept_opt,
                         workspace, (uint8_t*)pcache_dst, acc_dst, pos_dst, (hipStream_t)stream);
}

}  // extern "C"
