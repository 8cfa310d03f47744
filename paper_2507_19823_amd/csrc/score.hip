// Step 2: the key scan.  z~ = q . Q(K)^T (Eq. 2 / Eq. 3) for every resident token, streamed
// once from HBM as packed codes and contracted on the matrix cores in exact integer arithmetic.
#include "hca_internal.h"

namespace hca {

// Work split: grid.y = row, grid.x = chunk; a workgroup has 4 waves and each wave scans
// `bpw` consecutive 1 KiB code blocks.  U blocks are fetched ahead of use to keep several KiB
// per wave in flight.
template <int BITS, bool WRITE_Z, int U>
__global__ __launch_bounds__(256) void score_kernel(Layout L, const uint8_t* __restrict__ kcache,
                                                    const uint16_t* __restrict__ q, NRes nr, int bpw,
                                                    float* __restrict__ sel, float* __restrict__ z) {
  __shared__ QShared sh;
  const int row = blockIdx.y;
  const int64_t n = nr.n[row / L.n_kv_heads];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int64_t nblocks = (n + L.tpb - 1) / L.tpb;
  const int64_t wave_first = ((int64_t)blockIdx.x * 4 + w) * bpw;
  if ((int64_t)blockIdx.x * 4 * bpw >= nblocks) return;  // whole workgroup past the end
  load_query(q, row, L.gqa, L.group, &sh);
  QOperand<BITS> op;
  build_operand<BITS>(&sh, &op);
  int64_t wave_end = wave_first + bpw;
  if (wave_end > nblocks) wave_end = nblocks;

  const uint4* cbase = reinterpret_cast<const uint4*>(kcache + (int64_t)row * L.codes_row_bytes()) + lane;
  const uint8_t* mbase = kcache + L.meta_off + (int64_t)row * L.meta_row_bytes();
  const int t = lane & 15, hd = lane >> 4;
  float* selrow = sel + (int64_t)row * L.cap;
  float* zrow = WRITE_Z ? z + ((int64_t)row * L.gqa + hd) * L.cap : nullptr;

  for (int64_t b0 = wave_first; b0 < wave_end; b0 += U) {
    uint4 wv[U];
    uint4 mv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int64_t b = b0 + u;
      if (b >= wave_end) b = wave_end - 1;   // clamp: reload a valid block, result discarded
      wv[u] = cbase[b * 64];
      if (BITS == 4) {
        mv[u] = *reinterpret_cast<const uint4*>(mbase + b * kMetaBytes + t * 16);
      } else {                               // tokens t (tile 0) and 16+t (tile 1)
        const uint2 m0 = *reinterpret_cast<const uint2*>(mbase + b * kMetaBytes + t * 8);
        const uint2 m1 = *reinterpret_cast<const uint2*>(mbase + b * kMetaBytes + (16 + t) * 8);
        mv[u] = uint4{m0.x, m0.y, m1.x, m1.y};
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t b = b0 + u;
      if (b >= wave_end) break;
      if constexpr (BITS == 4) {
        const float zv = score_block4(op, wv[u], mv[u]);
        float best = (hd < L.gqa) ? zv : -INFINITY;
        best = fmaxf(best, __shfl_xor(best, 16));
        best = fmaxf(best, __shfl_xor(best, 32));
        const int64_t tok = b * 16 + t;
        if (tok < n) {
          if (hd == 0) selrow[tok] = best;
          if (WRITE_Z && hd < L.gqa) zrow[tok] = zv;
        }
      } else {
        const QOperand<2>& o2 = op;
        const float z0 = score_tile2(o2, wv[u].x, wv[u].y, uint2{mv[u].x, mv[u].y});
        const float z1 = score_tile2(o2, wv[u].z, wv[u].w, uint2{mv[u].z, mv[u].w});
        float b0v = (hd < L.gqa) ? z0 : -INFINITY;
        float b1v = (hd < L.gqa) ? z1 : -INFINITY;
        b0v = fmaxf(b0v, __shfl_xor(b0v, 16));
        b1v = fmaxf(b1v, __shfl_xor(b1v, 16));
        b0v = fmaxf(b0v, __shfl_xor(b0v, 32));
        b1v = fmaxf(b1v, __shfl_xor(b1v, 32));
        const int64_t tok0 = b * 32 + t, tok1 = tok0 + 16;
        if (tok0 < n) {
          if (hd == 0) selrow[tok0] = b0v;
          if (WRITE_Z && hd < L.gqa) zrow[tok0] = z0;
        }
        if (tok1 < n) {
          if (hd == 0) selrow[tok1] = b1v;
          if (WRITE_Z && hd < L.gqa) zrow[tok1] = z1;
        }
      }
    }
  }
}

int32_t launch_score(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax,
                     float* sel, float* z_opt, hipStream_t st) {
  if (nmax == 0) return HCA_OK;
  const int64_t nblocks = (nmax + L.tpb - 1) / L.tpb;
  // aim at ~16 waves per SIMD over the whole chip when the cache is large, >= 4 blocks per wave
  const int64_t total = nblocks * L.rows;
  const Tuning& tn = tuning();
  int64_t bpw = total / (256 * 4 * 16);
  if (bpw < 4) bpw = 4;
  if (bpw > 32) bpw = 32;
  if (tn.score_bpw > 0) bpw = tn.score_bpw;
  dim3 grid((unsigned)((nblocks + 4 * bpw - 1) / (4 * bpw)), (unsigned)L.rows);
  const uint8_t* kc = (const uint8_t*)kcache;
  const uint16_t* qq = (const uint16_t*)q;
#define HCA_SCORE(B, Z, U) score_kernel<B, Z, U><<<grid, 256, 0, st>>>(L, kc, qq, nr, (int)bpw, sel, z_opt)
#define HCA_SCORE_U(B, Z)                                  \
  do {                                                     \
    if (tn.score_depth >= 8) HCA_SCORE(B, Z, 8);           \
    else if (tn.score_depth >= 4) HCA_SCORE(B, Z, 4);      \
    else HCA_SCORE(B, Z, 2);                               \
  } while (0)
  if (L.bits == 4) {
    if (z_opt) HCA_SCORE_U(4, true); else HCA_SCORE_U(4, false);
  } else {
    if (z_opt) HCA_SCORE_U(2, true); else HCA_SCORE_U(2, false);
  }
#undef HCA_SCORE_U
#undef HCA_SCORE
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

}  // namespace hca
