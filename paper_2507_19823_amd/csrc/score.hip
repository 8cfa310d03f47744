// Step 2: the key scan.  z~ = q . Q(K)^T (Eq. 2 / Eq. 3) for every resident token, streamed
// once from HBM as packed codes and contracted on the matrix cores in exact integer arithmetic.
#include "hca_internal.h"

namespace hca {

// max of two finite floats (plain v_max_f32: the inputs are never NaN, so no canonicalisation)
__device__ __forceinline__ float fmax_raw(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

// max over the four 16-lane rows of a wave (the four query heads of a token), result on every lane
__device__ __forceinline__ float max_over_heads(float x) {
  const uint32_t xi = __float_as_uint(x);
  const auto r16 = __builtin_amdgcn_permlane16_swap(xi, xi, false, false);   // rows {0,1} and {2,3}
  const float m = fmax_raw(__uint_as_float(r16[0]), __uint_as_float(r16[1]));
  const uint32_t mi = __float_as_uint(m);
  const auto r32 = __builtin_amdgcn_permlane32_swap(mi, mi, false, false);   // halves
  return fmax_raw(__uint_as_float(r32[0]), __uint_as_float(r32[1]));
}

// 16-byte load with the non-temporal hint: the code stream is read once per decode step and
// should not displace anything in the caches.
__device__ __forceinline__ uint4 load_stream16(const uint4* p) {
  const v4i v = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(p));
  return uint4{(uint32_t)v.x, (uint32_t)v.y, (uint32_t)v.z, (uint32_t)v.w};
}

// All-gather over the four 16-lane rows of a wave: returns, on every lane, the values that the
// lanes of the same column hold in rows 0..3.
__device__ __forceinline__ uint4 allgather_rows(uint32_t v) {
  const auto a = __builtin_amdgcn_permlane16_swap(v, v, false, false);        // [r0 r0 r2 r2], [r1 r1 r3 r3]
  const auto b = __builtin_amdgcn_permlane32_swap(a[0], a[0], false, false);  // r0 everywhere, r2 everywhere
  const auto c = __builtin_amdgcn_permlane32_swap(a[1], a[1], false, false);  // r1 everywhere, r3 everywhere
  return uint4{b[0], c[0], b[1], c[1]};
}

// Work split: grid.y = row, grid.x = chunk; a workgroup has 4 waves and each wave scans `bpw`
// consecutive 1 KiB code blocks, U at a time: U code loads (16 B per lane, the lane's own MFMA
// operand bytes) and U meta loads (4 B per lane, then an all-gather over the four lanes of a
// token) are issued before the first block is scored, and the selection scores of four 16-token
// tiles leave in one 256-byte store.  Block indices are wave-uniform (scalar registers).
// LSE: every wave also leaves, per query head, the (max, sum of exp) pair of its logits z~ * sm_scale
// in `part` ([row][4][waves of the row] float2), from which lse_merge forms the softmax denominator
// over all resident tokens.
template <int BITS, bool WRITE_Z, int U, bool LSE = false>
__global__ __launch_bounds__(256) void score_kernel(Layout L, const uint8_t* __restrict__ kcache,
                                                    const uint16_t* __restrict__ q, NRes nr, int bpw,
                                                    float* __restrict__ sel, float* __restrict__ z,
                                                    uint64_t* __restrict__ stamps, float sm_scale = 0.f,
                                                    float2* __restrict__ part = nullptr) {
  static_assert(U % 4 == 0, "stores are batched four tiles at a time");
  __shared__ QShared sh;
  const int row = blockIdx.y;
  const int64_t n = nr.n[row / L.n_kv_heads];
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nblocks = (int)((n + L.tpb - 1) / L.tpb);
  if ((int64_t)blockIdx.x * 4 * bpw >= nblocks) return;  // whole workgroup past the end
  // optional profiling: every wave leaves its start and end time (constant-rate wall clock)
  uint64_t* stamp = stamps ? stamps + (((int64_t)row * gridDim.x + blockIdx.x) * 4 + w) * 2 : nullptr;
  if (stamp && lane == 0) stamp[0] = wall_clock64();
  const int wave_first = (blockIdx.x * 4 + w) * bpw;
  int wave_end = wave_first + bpw;
  if (wave_end > nblocks) wave_end = nblocks;
  if (wave_end < wave_first) wave_end = wave_first;

  QOperand<BITS> op;                          // filled in after the first loads are in flight
  const int t = lane & 15, hd = lane >> 4;
  const uint4* cptr = reinterpret_cast<const uint4*>(kcache + (int64_t)row * L.codes_row_bytes()) + lane;
  // this lane's dword of a 256-byte meta block: 4-bit: dword hd of token t (16 B per token);
  // 2-bit: dword hd&1 of token 16*(hd>>1) + t (8 B per token)
  const uint32_t* mptr = reinterpret_cast<const uint32_t*>(kcache + L.meta_off + (int64_t)row * L.meta_row_bytes()) +
                         (BITS == 4 ? 4 * t + hd : 2 * (16 * (hd >> 1) + t) + (hd & 1));
  float* selrow = sel + (int64_t)row * L.cap;
  float* zrow = WRITE_Z ? z + ((int64_t)row * L.gqa + hd) * L.cap + t : nullptr;
  const bool head_live = hd < L.gqa;
  const int ntok = (int)n;
  // LSE: running max and sum of 2^(logit - max) of this lane's logits, in units of log2 (one multiply by
  // sm_scale * log2(e)); branch-free, raw v_exp_f32 (accurate to ~1 ulp here).
  float lm = -INFINITY, ls = 0.f;
  const float sm2 = sm_scale * 1.44269504f;
  auto lse_add = [&](float zv, bool valid) {
    const float l = valid ? zv * sm2 : -INFINITY;
    const float nm = fmaxf(lm, l);
    const float base = (nm == -INFINITY) ? 0.f : nm;        // nothing valid yet: both terms are 2^-inf = 0
    ls = fmaf(ls, __builtin_amdgcn_exp2f(lm - base), __builtin_amdgcn_exp2f(l - base));
    lm = nm;
  };
  auto lse_fold = [&]() {};
  // scores block b; returns the per-token max over heads of its tile(s) (on every lane)
  auto score_one = [&](int b, uint4 wv, uint32_t mword, float& best0, float& best1) {
    const uint4 mv = allgather_rows(mword);
    if constexpr (BITS == 4) {
      const float zv = score_block4(op, wv, mv);
      best0 = max_over_heads(head_live ? zv : -INFINITY);
      best1 = best0;
      if (WRITE_Z && head_live && b * 16 + t < ntok) zrow[b * 16] = zv;
      if constexpr (LSE) lse_add(zv, head_live && b * 16 + t < ntok);
    } else {
      const float z0 = score_tile2(op, wv.x, wv.y, uint2{mv.x, mv.y});
      const float z1 = score_tile2(op, wv.z, wv.w, uint2{mv.z, mv.w});
      best0 = max_over_heads(head_live ? z0 : -INFINITY);
      best1 = max_over_heads(head_live ? z1 : -INFINITY);
      if (WRITE_Z && head_live) {
        if (b * 32 + t < ntok) zrow[b * 32] = z0;
        if (b * 32 + 16 + t < ntok) zrow[b * 32 + 16] = z1;
      }
      if constexpr (LSE) {
        lse_add(z0, head_live && b * 32 + t < ntok);
        lse_add(z1, head_live && b * 32 + 16 + t < ntok);
      }
    }
  };
  // the lane in row hd stores tile hd of four consecutive tiles starting at token tok0
  auto store4 = [&](int tok0, float v0, float v1, float v2, float v3) {
    const float v = hd == 0 ? v0 : (hd == 1 ? v1 : (hd == 2 ? v2 : v3));
    const int tok = tok0 + lane;                          // 16*hd + t == lane
    if (tok < ntok) selrow[tok] = v;
  };

  // Software pipeline over groups of U blocks: the loads of group g+1 are issued before group g is
  // scored and stored.  Loads and stores retire through one in-order counter, so a wait for a load
  // issued after a store would also wait for that store's acknowledgement; issuing the next loads
  // first keeps every store younger than the loads the wave waits for.
  auto fetch = [&](int g0, uint4 (&wv)[U], uint32_t (&mw)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      wv[u] = load_stream16(&cptr[(int64_t)(g0 + u) * 64]);
      mw[u] = __builtin_nontemporal_load(&mptr[(int64_t)(g0 + u) * 64]);
    }
  };
  auto consume = [&](int g0, const uint4 (&wv)[U], const uint32_t (&mw)[U]) {
    float lo[U], hi[U];
#pragma unroll
    for (int u = 0; u < U; ++u) score_one(g0 + u, wv[u], mw[u], lo[u], hi[u]);
    if constexpr (BITS == 4) {
#pragma unroll
      for (int u = 0; u < U; u += 4) store4((g0 + u) * 16, lo[u], lo[u + 1], lo[u + 2], lo[u + 3]);
    } else {
#pragma unroll
      for (int u = 0; u < U; u += 2) store4((g0 + u) * 32, lo[u], hi[u], lo[u + 1], hi[u + 1]);
    }
    if constexpr (LSE) lse_fold();
  };
  int b0 = wave_first;
  const int ngroups = (wave_end - wave_first) / U;
  uint4 wa[U], wb[U];
  uint32_t ma[U], mb[U];
  if (ngroups > 0) fetch(b0, wa, ma);        // first loads go out before the query is prepared
  load_query(q, row, L.gqa, L.group, &sh);
  build_operand<BITS>(&sh, &op);
  if (ngroups > 0) {
    int g = 0;
    for (; g + 2 <= ngroups; g += 2) {
      fetch(b0 + U, wb, mb);
      consume(b0, wa, ma);
      if (g + 2 < ngroups) fetch(b0 + 2 * U, wa, ma);
      consume(b0 + U, wb, mb);
      b0 += 2 * U;
    }
    if (g < ngroups) {          // odd group count: the last group is already in wa / ma
      consume(b0, wa, ma);
      b0 += U;
    }
  }
  for (; b0 < wave_end; ++b0) {              // tail: one block at a time
    const uint4 wv = load_stream16(&cptr[(int64_t)b0 * 64]);
    const uint32_t mw = __builtin_nontemporal_load(&mptr[(int64_t)b0 * 64]);
    float lo, hi;
    score_one(b0, wv, mw, lo, hi);
    if constexpr (LSE) lse_fold();
    if constexpr (BITS == 4) {
      if (hd == 0 && b0 * 16 + t < ntok) selrow[b0 * 16 + t] = lo;
    } else {
      if (hd == 0 && b0 * 32 + t < ntok) selrow[b0 * 32 + t] = lo;
      if (hd == 1 && b0 * 32 + 16 + t < ntok) selrow[b0 * 32 + 16 + t] = hi;
    }
  }
  if constexpr (LSE) {
    // merge over the 16 lanes of a head row, then one lane per head stores the wave's pair
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) {
      const float om = __shfl_xor(lm, o), os = __shfl_xor(ls, o);
      const float mm = fmaxf(lm, om);
      const float bs = (mm == -INFINITY) ? 0.f : mm;
      ls = ls * __builtin_amdgcn_exp2f(lm - bs) + os * __builtin_amdgcn_exp2f(om - bs);
      lm = mm;
    }
    if (t == 0)   // back to natural-log units: max in logit units, the sum is unit-free
      part[((int64_t)row * 4 + hd) * (gridDim.x * 4) + blockIdx.x * 4 + w] = float2{lm * 0.693147181f, ls};
  }
  if (stamp && lane == 0) stamp[1] = wall_clock64();
}

// lse[row * G + h] = log sum exp over the first `live` wave pairs of the row (waves of workgroups that
// returned at once wrote nothing); -inf for a row without resident tokens.
__global__ __launch_bounds__(256) void lse_merge(Layout L, NRes nr, int bpw, int waves_per_row,
                                                 const float2* __restrict__ part, float* __restrict__ lse) {
  __shared__ float sm[4], ss[4];
  const int row = blockIdx.x / L.gqa, h = blockIdx.x % L.gqa;
  const int64_t n = nr.n[row / L.n_kv_heads];
  const int64_t nblocks = (n + L.tpb - 1) / L.tpb;
  const int64_t live_wgs = (nblocks + 4 * bpw - 1) / (4 * bpw);
  const int live = (int)(live_wgs * 4);
  const float2* p = part + ((int64_t)row * 4 + h) * waves_per_row;
  float m = -INFINITY, s = 0.f;
  for (int i = threadIdx.x; i < live; i += 256) {
    const float2 v = p[i];
    if (v.x != -INFINITY) {
      const float mm = fmaxf(m, v.x);
      s = (m == -INFINITY ? 0.f : s * expf(m - mm)) + v.y * expf(v.x - mm);
      m = mm;
    }
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const float om = __shfl_xor(m, o), os = __shfl_xor(s, o);
    const float mm = fmaxf(m, om);
    s = (m == -INFINITY ? 0.f : s * expf(m - mm)) + (om == -INFINITY ? 0.f : os * expf(om - mm));
    m = mm;
  }
  if ((threadIdx.x & 63) == 0) { sm[threadIdx.x >> 6] = m; ss[threadIdx.x >> 6] = s; }
  __syncthreads();
  if (threadIdx.x == 0) {
    float M = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
    float S = 0.f;
    for (int x = 0; x < 4; ++x) if (sm[x] != -INFINITY) S += ss[x] * expf(sm[x] - M);
    lse[blockIdx.x] = (M == -INFINITY) ? -INFINITY : M + logf(S);
  }
}

// number of (start, end) stamp pairs a scan launch over nmax tokens writes at most
int64_t score_stamp_pairs(const Layout& L, int64_t nmax) {
  const int64_t nblocks = (nmax + L.tpb - 1) / L.tpb;
  return (nblocks / 4 + 1) * 4 * L.rows;      // >= grid.x * 4 waves * rows for any blocks-per-wave >= 4
}

// float2 pairs a scan launch with LSE leaves per row: 4 heads x (waves of the row), for any blocks-per-wave >= 4
size_t score_workspace_bytes(const Layout& L) {
  return (size_t)L.rows * 4 * (size_t)(L.nblk / 4 + 8) * sizeof(float2);
}

int32_t launch_score(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax,
                     float* sel, float* z_opt, hipStream_t st, uint64_t* stamps) {
  if (nmax == 0) return HCA_OK;
  const int64_t nblocks = (nmax + L.tpb - 1) / L.tpb;
  // aim at ~16 waves per SIMD over the whole chip when the cache is large, >= 4 blocks per wave
  const int64_t total = nblocks * L.rows;
  const Tuning& tn = tuning();
  int64_t bpw = total / (256 * 4 * 16);
  if (bpw < 4) bpw = 4;
  // measured best on MI355X: 4-bit codes 8 blocks ahead, 16 per wave; 2-bit codes (two tiles per block,
  // more registers) 4 ahead, 32 per wave
  const int64_t bpw_max = L.bits == 4 ? 16 : 32;
  if (bpw > bpw_max) bpw = bpw_max;
  if (tn.score_bpw > 0) bpw = tn.score_bpw;
  const int depth = tn.score_depth > 0 ? tn.score_depth : (L.bits == 4 ? 8 : 4);
  dim3 grid((unsigned)((nblocks + 4 * bpw - 1) / (4 * bpw)), (unsigned)L.rows);
  const uint8_t* kc = (const uint8_t*)kcache;
  const uint16_t* qq = (const uint16_t*)q;
#define HCA_SCORE(B, Z, U) score_kernel<B, Z, U><<<grid, 256, 0, st>>>(L, kc, qq, nr, (int)bpw, sel, z_opt, stamps)
#define HCA_SCORE_U(B, Z)                                  \
  do {                                                     \
    if (depth >= 8) HCA_SCORE(B, Z, 8);                    \
    else HCA_SCORE(B, Z, 4);                               \
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

// The scan with the softmax denominator over all resident tokens as a second output (no z output, no stamps).
int32_t launch_score_lse(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax,
                         float sm_scale, float* sel, float* lse_out, void* lse_ws, hipStream_t st) {
  if (nmax == 0) {
    lse_merge<<<L.rows * L.gqa, 256, 0, st>>>(L, nr, 4, 0, nullptr, lse_out);
    HCA_HIP(hipGetLastError());
    return HCA_OK;
  }
  const int64_t nblocks = (nmax + L.tpb - 1) / L.tpb;
  const int64_t total = nblocks * L.rows;
  const Tuning& tn = tuning();
  int64_t bpw = total / (256 * 4 * 16);
  if (bpw < 4) bpw = 4;
  const int64_t bpw_max = L.bits == 4 ? 16 : 32;
  if (bpw > bpw_max) bpw = bpw_max;
  if (tn.score_bpw >= 4) bpw = tn.score_bpw;
  dim3 grid((unsigned)((nblocks + 4 * bpw - 1) / (4 * bpw)), (unsigned)L.rows);
  if ((size_t)L.rows * 4 * grid.x * 4 * sizeof(float2) > score_workspace_bytes(L)) return HCA_ERR_CAPACITY;
  const uint8_t* kc = (const uint8_t*)kcache;
  const uint16_t* qq = (const uint16_t*)q;
  float2* part = (float2*)lse_ws;
  // 4 blocks ahead instead of 8: the extra running state would otherwise cost a wave of occupancy per SIMD
  if (L.bits == 4)
    score_kernel<4, false, 4, true><<<grid, 256, 0, st>>>(L, kc, qq, nr, (int)bpw, sel, nullptr, nullptr, sm_scale, part);
  else
    score_kernel<2, false, 4, true><<<grid, 256, 0, st>>>(L, kc, qq, nr, (int)bpw, sel, nullptr, nullptr, sm_scale, part);
  lse_merge<<<L.rows * L.gqa, 256, 0, st>>>(L, nr, (int)bpw, (int)grid.x * 4, part, lse_out);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

}  // namespace hca
