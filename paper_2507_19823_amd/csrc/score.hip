// Step 2: the key scan.  z~ = q . Q(K)^T (Eq. 2 / Eq. 3) for every resident token, streamed
// once from HBM as packed codes and contracted on the matrix cores in exact integer arithmetic.
#include <math.h>
#include <stdlib.h>

#include "hca_internal.h"
#include "quantize_device.h"

namespace hca {

struct NRes32 { int32_t n[kMaxBatch]; };   // row lengths as kernel arguments of the paired launches

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

// The same all-gather through the LDS crossbar (ds_bpermute_b32: no LDS memory is touched): four reads with the
// byte addresses of lanes column + 16 r, r = 0..3.  The scan is bound by vector-ALU issue, the LDS pipe is idle.
struct RowGather {
  int a0, a1, a2, a3;
  __device__ __forceinline__ explicit RowGather(int lane) {
    a0 = 4 * (lane & 15); a1 = a0 + 64; a2 = a0 + 128; a3 = a0 + 192;
  }
  __device__ __forceinline__ uint4 operator()(uint32_t v) const {
    return uint4{(uint32_t)__builtin_amdgcn_ds_bpermute(a0, (int)v), (uint32_t)__builtin_amdgcn_ds_bpermute(a1, (int)v),
                 (uint32_t)__builtin_amdgcn_ds_bpermute(a2, (int)v), (uint32_t)__builtin_amdgcn_ds_bpermute(a3, (int)v)};
  }
};

// Four values per lane, one per 16-token tile (z0..z3: the score of this lane's (token, head) in tiles 0..3): returns,
// on the lanes of row r, the maximum over the four rows (= the token's four query heads) of tile r's values - the
// reduction and the hand-over of tile r to row r in three swaps and three maxima.
__device__ __forceinline__ float max_over_heads_scatter(float z0, float z1, float z2, float z3) {
  const auto p = __builtin_amdgcn_permlane32_swap(__float_as_uint(z0), __float_as_uint(z2), false, false);
  const auto q = __builtin_amdgcn_permlane32_swap(__float_as_uint(z1), __float_as_uint(z3), false, false);
  // p[0] = [z0.r0 z0.r1 z2.r0 z2.r1], p[1] = [z0.r2 z0.r3 z2.r2 z2.r3]: maxima over the row pairs (0,2), (1,3)
  const float m02 = fmax_raw(__uint_as_float(p[0]), __uint_as_float(p[1]));
  const float m13 = fmax_raw(__uint_as_float(q[0]), __uint_as_float(q[1]));
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(m02), __float_as_uint(m13), false, false);
  // r[0] = [m02.r0 m13.r0 m02.r2 m13.r2], r[1] = [m02.r1 m13.r1 m02.r3 m13.r3]
  return fmax_raw(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// The float whose order key is `key`, or -inf for keys below those of all finite floats (0: "no threshold"):
// v >= key_floor(key) <=> order_key(v) >= key for every finite v (-0 and +0 share a key and compare equal).
__device__ __forceinline__ float key_floor(uint32_t key) {
  if (key <= 0x007fffffu) return -INFINITY;
  return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}

// Work split: grid.y = row, grid.x = chunk; a workgroup has 4 waves and each wave scans `bpw`
// consecutive 1 KiB code blocks, U at a time: U code loads (16 B per lane, the lane's own MFMA
// operand bytes) and U meta loads (4 B per lane, then an all-gather over the four lanes of a
// token) are issued before the first block is scored, and the selection scores of four 16-token
// tiles leave in one 256-byte store.  Block indices are wave-uniform (scalar registers).
// LSE: every wave also leaves, per query head, the (max, sum of exp) pair of its logits z~ * sm_scale
// in `part` ([row][4][waves of the row] float2), from which lse_merge forms the softmax denominator
// over all resident tokens.
// SELECT: instead of the score of every token, only the (order key, slot) pairs of the tokens whose key reaches the
// row's threshold t0 leave the kernel, in slot order, as the list of the workgroup's chunk (chunk = the slots of
// one workgroup; chunk c of a row owns entries [c * chunk, (c + 1) * chunk) of the row's list area, so no two
// workgroups ever contend for a position and no workgroup waits for an atomic).  With a threshold a little below the k-th largest
// score of the row the 4 bytes per token of score traffic - written here and read twice by the top-k passes -
// shrink to a few thousand pairs per row.
// bx = the workgroup's chunk of the row, gx = chunks per row (blockIdx.x and gridDim.x in the plain launch)
template <int BITS, bool WRITE_Z, int U, bool LSE, bool SELECT>
__device__ __forceinline__ void score_body(const Layout& L, const uint8_t* __restrict__ kcache,
                                           const uint16_t* __restrict__ q, const int64_t n, int bpw,
                                           float* __restrict__ sel, float* __restrict__ z,
                                           uint64_t* __restrict__ stamps, float sm_scale, float2* __restrict__ part,
                                           const SelectOut& so, const int bx, const int gx, const int row) {
  static_assert(U % 4 == 0, "stores are batched four tiles at a time");
  __shared__ QShared sh;
  // SELECT: every wave collects its qualifying pairs in slot order in its quarter of the dynamic LDS (room for
  // all the wave's slots), then the workgroup strings the four lists together
  extern __shared__ uint2 wlist_all[];
  __shared__ uint32_t wcount[8];
  __shared__ __align__(16) uint32_t opimg[64 * 8];
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nblocks = (int)((n + L.tpb - 1) / L.tpb);
  if ((int64_t)bx * 4 * bpw >= nblocks) {        // whole workgroup past the end
    if (SELECT && threadIdx.x == 0) {
      so.ncand[(int64_t)row * kSelectMaxChunks + bx] = 0;
      so.n1[(int64_t)row * kSelectMaxChunks + bx] = 0;
    }
    return;
  }
  // optional profiling: every wave leaves its start and end time (constant-rate wall clock)
  uint64_t* stamp = stamps ? stamps + (((int64_t)row * gx + bx) * 4 + w) * 2 : nullptr;
  if (stamp && lane == 0) stamp[0] = wall_clock64();
  const int wave_first = (bx * 4 + w) * bpw;
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
  const RowGather gather_rows(lane);
  // scores block b: this lane's (token, head) score of the block's tile (4-bit) or two tiles (2-bit); -inf on the
  // lanes of query heads that do not exist
  auto score_one = [&](int b, uint4 wv, uint4 mv, float& zt0, float& zt1) {
    if constexpr (BITS == 4) {
      const float zv = score_block4(op, wv, mv);
      zt0 = head_live ? zv : -INFINITY;
      if (WRITE_Z && head_live && b * 16 + t < ntok) zrow[b * 16] = zv;
      if constexpr (LSE) lse_add(zv, head_live && b * 16 + t < ntok);
    } else {
      const float z0 = score_tile2(op, wv.x, wv.y, uint2{mv.x, mv.y});
      const float z1 = score_tile2(op, wv.z, wv.w, uint2{mv.z, mv.w});
      zt0 = head_live ? z0 : -INFINITY;
      zt1 = head_live ? z1 : -INFINITY;
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
  const uint32_t t0key = SELECT ? so.spec[4 * row] : 0u;
  const uint32_t t1key = SELECT ? so.spec[4 * row + 2] : 0u;   // the deeper threshold: only counted against
  const float t0f = key_floor(t0key), t1f = key_floor(t1key);  // the same thresholds as floats: one compare each
  uint32_t n1 = 0;                                         // slots of this wave with key >= t1key (wave-uniform)
  uint2* wlist = SELECT ? wlist_all + (int64_t)w * bpw * L.tpb : nullptr;
  uint32_t nlist = 0;                                     // SELECT: pairs in this wave's list so far (wave-uniform)
  // SELECT: appends the lanes' pairs that qualify, in lane order (the caller's lanes are in slot order)
  auto emit_pairs = [&](float v, int tok, bool live) {
    n1 += (uint32_t)__popcll(__builtin_amdgcn_ballot_w64(live && v >= t1f));
    const bool hit = live && v >= t0f;
    const uint64_t m = __builtin_amdgcn_ballot_w64(hit);
    if (m != 0) {
      if (hit) wlist[nlist + (uint32_t)__popcll(m & ((1ull << lane) - 1))] = uint2{order_key(v), (uint32_t)tok};
      nlist += (uint32_t)__popcll(m);
    }
  };
  // four consecutive tiles starting at token tok0, this lane's (token, head) score in each: the lanes of row r end
  // up with tile r's selection score (maximum over the heads), i.e. lane l with that of token tok0 + l
  auto store4 = [&](int tok0, float z0, float z1, float z2, float z3) {
    const float v = max_over_heads_scatter(z0, z1, z2, z3);
    const int tok = tok0 + lane;                          // 16*hd + t == lane
    if constexpr (SELECT) emit_pairs(v, tok, tok < ntok);
    else if (tok < ntok) selrow[tok] = v;
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
    // the meta all-gather runs two blocks ahead of the scoring (its results come back through the LDS queue); the
    // scheduling fences keep it there - all U gathers issued at once cost a wave of occupancy in registers
    uint4 mv0 = gather_rows(mw[0]);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint4 mv = mv0;
      if (u + 1 < U) mv0 = gather_rows(mw[u + 1]);
      score_one(g0 + u, wv[u], mv, lo[u], hi[u]);
      if constexpr (BITS == 4) asm volatile("" : "+v"(lo[u]));
      else asm volatile("" : "+v"(lo[u]), "+v"(hi[u]));
    }
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
  build_operand_shared<BITS>(&sh, opimg, &op);
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
    score_one(b0, wv, gather_rows(mw), lo, hi);
    lo = max_over_heads(lo);
    if constexpr (BITS == 2) hi = max_over_heads(hi);
    if constexpr (LSE) lse_fold();
    if constexpr (SELECT) {
      // lanes 0..15 carry tile 0; with 2-bit codes lanes 16..31 carry tile 1: lane order is slot order
      if constexpr (BITS == 4) emit_pairs(lo, b0 * 16 + t, hd == 0 && b0 * 16 + t < ntok);
      else emit_pairs(hd == 0 ? lo : hi, b0 * 32 + 16 * hd + t, hd < 2 && b0 * 32 + 16 * hd + t < ntok);
    } else if constexpr (BITS == 4) {
      if (hd == 0 && b0 * 16 + t < ntok) selrow[b0 * 16 + t] = lo;
    } else {
      if (hd == 0 && b0 * 32 + t < ntok) selrow[b0 * 32 + t] = lo;
      if (hd == 1 && b0 * 32 + 16 + t < ntok) selrow[b0 * 32 + 16 + t] = hi;
    }
  }
  if constexpr (SELECT) {
    // the four waves' lists, in wave order (= slot order), become the chunk's list
    if (lane == 0) { wcount[w] = nlist; wcount[4 + w] = n1; }
    __syncthreads();
    uint32_t base = 0, total = 0;
#pragma unroll
    for (int x = 0; x < 4; ++x) { if (x < w) base += wcount[x]; total += wcount[x]; }
    const int64_t chunk_slots = (int64_t)4 * bpw * L.tpb;
    uint2* dst = so.lists + (int64_t)row * so.row_entries + (int64_t)bx * chunk_slots + base;
    for (uint32_t i = lane; i < nlist; i += 64) dst[i] = wlist[i];
    if (threadIdx.x == 0) {
      so.ncand[(int64_t)row * kSelectMaxChunks + bx] = total;
      so.n1[(int64_t)row * kSelectMaxChunks + bx] = wcount[4] + wcount[5] + wcount[6] + wcount[7];
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
      part[((int64_t)row * 4 + hd) * (gx * 4) + bx * 4 + w] = float2{lm * 0.693147181f, ls};
  }
  if (stamp && lane == 0) stamp[1] = wall_clock64();
}

template <int BITS, bool WRITE_Z, int U, bool LSE = false, bool SELECT = false>
__global__ __launch_bounds__(256) void score_kernel(Layout L, const uint8_t* __restrict__ kcache,
                                                    const uint16_t* __restrict__ q, NRes nr, int bpw,
                                                    float* __restrict__ sel, float* __restrict__ z,
                                                    uint64_t* __restrict__ stamps, float sm_scale = 0.f,
                                                    float2* __restrict__ part = nullptr, SelectOut so = SelectOut{}) {
  score_body<BITS, WRITE_Z, U, LSE, SELECT>(L, kcache, q, nr.n[blockIdx.y / L.n_kv_heads], bpw, sel, z, stamps, sm_scale,
                                            part, so, (int)blockIdx.x, (int)gridDim.x, (int)blockIdx.y);
}

// The selecting scan as a launch of its own (hca_score_topk): registers capped for four waves per SIMD.
template <int BITS, int U>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4))) void score_select_kernel(
    Layout L, const uint8_t* __restrict__ kcache, const uint16_t* __restrict__ q, NRes nr, int bpw,
    uint64_t* __restrict__ stamps, SelectOut so) {
  score_body<BITS, false, U, false, true>(L, kcache, q, nr.n[blockIdx.y / L.n_kv_heads], bpw, nullptr, nullptr, stamps,
                                          0.f, nullptr, so, (int)blockIdx.x, (int)gridDim.x, (int)blockIdx.y);
}

// The selecting scan once more for the rows whose sampled threshold left too few pairs (spec[row][1] != 0, with
// the threshold already reset to 0).  Almost always there is no such row, so the launch is kept small - up to 256
// workgroups per row that walk over the row's chunks - and costs next to nothing when it has nothing to do.
template <int BITS, int U>
__global__ __launch_bounds__(256) void score_failed_rows_kernel(Layout L, const uint8_t* __restrict__ kcache,
                                                                const uint16_t* __restrict__ q, NRes nr, int bpw,
                                                                int nchunks, SelectOut so) {
  if (so.spec[4 * blockIdx.y + 1] == 0) return;
  for (int bx = blockIdx.x; bx < nchunks; bx += gridDim.x) {
    score_body<BITS, false, U, false, true>(L, kcache, q, nr.n[blockIdx.y / L.n_kv_heads], bpw, nullptr, nullptr, nullptr,
                                            0.f, nullptr, so, bx, nchunks, (int)blockIdx.y);
    __syncthreads();                                        // the shared query image and counters are reused
  }
}

// The same for the two layers of a paired launch: grid.y = 2 x rows.
struct RescanSide {
  const uint8_t* kcache;
  const uint16_t* q;
  SelectOut so;
  int32_t bpw, nchunks;
  NRes32 nr;
};
template <int BITS, int U>
__device__ __forceinline__ void rescan_side(const Layout& L, const RescanSide& s, const int row) {
  if (s.so.spec[4 * row + 1] == 0) return;
  for (int bx = blockIdx.x; bx < s.nchunks; bx += gridDim.x) {
    score_body<BITS, false, U, false, true>(L, s.kcache, s.q, s.nr.n[row / L.n_kv_heads], s.bpw, nullptr, nullptr, nullptr,
                                            0.f, nullptr, s.so, bx, s.nchunks, row);
    __syncthreads();
  }
}
template <int BITS, int U>
__global__ __launch_bounds__(256) void score_failed_rows_pair_kernel(Layout L, RescanSide a, RescanSide b) {
  if ((int)blockIdx.y < L.rows) rescan_side<BITS, U>(L, a, (int)blockIdx.y);
  else rescan_side<BITS, U>(L, b, (int)blockIdx.y - L.rows);
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

// Threshold estimate for the selecting scan.  m slots of every row (whole code blocks, evenly spaced: sampled
// block s is block floor(s * nblocks / S) of the row, S = min(nblocks, m / slots per block); m = 8192 .. 65536, a
// power of two chosen by select_sample_count) are scored by select_sample_score; select_sample_rank
// then leaves in spec[row] a key t0 such that, if the sample behaves like a random one, at least `want` slots of
// the row have keys >= t0 with overwhelming probability:
//   m = sampled slots, kappa = want * m / n, r = ceil((3 + sqrt(9 + kappa))^2)  (the count of slots above the
//   r-th largest of m samples has mean n r / m and deviation n sqrt(r) / m: this r puts `want` six deviations
//   below the mean), t0 = the r-th largest sampled key with its low 10 bits cleared; t0 = 0 when r >= m.
// The selection stays exact whatever the sample does: a row whose list comes out short is scanned again with
// t0 = 0 (spec[row][1]).
constexpr int kSamplePerWg = 512;       // sampled slots per workgroup: m / 512 workgroups per row

// bx = which of the m / kSamplePerWg workgroups of the row this is; called by all 256 threads
template <int BITS>
__device__ __forceinline__ void sample_score_body(const Layout& L, const uint8_t* __restrict__ kcache,
                                                  const uint16_t* __restrict__ q, const int64_t n,
                                                  uint32_t* __restrict__ samples, const int m, const int bx,
                                                  const int row) {
  constexpr int kTpb = BITS == 4 ? 16 : 32;
  constexpr int kPerWave = kSamplePerWg / kTpb / 4;        // sampled blocks per wave: 8 (4-bit) or 4
  __shared__ QShared sh;
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (n <= 0) {                                             // nothing to sample: this workgroup's share reads "no slot"
    for (int i = threadIdx.x; i < kSamplePerWg; i += 256)
      samples[(int64_t)row * m + bx * kSamplePerWg + i] = 0;
    return;
  }
  const int nblocks = (int)((n + kTpb - 1) / kTpb);
  const int S = nblocks < m / kTpb ? nblocks : m / kTpb;
  const int t = lane & 15, hd = lane >> 4;
  const uint4* cptr = reinterpret_cast<const uint4*>(kcache + (int64_t)row * L.codes_row_bytes()) + lane;
  const uint32_t* mptr = reinterpret_cast<const uint32_t*>(kcache + L.meta_off + (int64_t)row * L.meta_row_bytes()) +
                         (BITS == 4 ? 4 * t + hd : 2 * (16 * (hd >> 1) + t) + (hd & 1));
  uint32_t* out = samples + (int64_t)row * m;
  const int s0 = (bx * 4 + w) * kPerWave;
  uint4 wv[kPerWave];
  uint32_t mw[kPerWave];
  int blk[kPerWave];
#pragma unroll
  for (int u = 0; u < kPerWave; ++u) {
    const int s = s0 + u;
    blk[u] = s < S ? (int)((int64_t)s * nblocks / S) : 0;
    wv[u] = load_stream16(&cptr[(int64_t)blk[u] * 64]);
    mw[u] = __builtin_nontemporal_load(&mptr[(int64_t)blk[u] * 64]);
  }
  QOperand<BITS> op;
  load_query(q, row, L.gqa, L.group, &sh);
  build_operand<BITS>(&sh, &op);
  const bool head_live = hd < L.gqa;
#pragma unroll
  for (int u = 0; u < kPerWave; ++u) {
    const int s = s0 + u;
    const uint4 mv = allgather_rows(mw[u]);
    if constexpr (BITS == 4) {
      const float zv = score_block4(op, wv[u], mv);
      const float best = max_over_heads(head_live ? zv : -INFINITY);
      const bool live = s < S && (int64_t)blk[u] * 16 + t < n;
      if (hd == 0) out[s * 16 + t] = live ? order_key(best) : 0u;      // no finite score has key 0
    } else {
      const float z0 = score_tile2(op, wv[u].x, wv[u].y, uint2{mv.x, mv.y});
      const float z1 = score_tile2(op, wv[u].z, wv[u].w, uint2{mv.z, mv.w});
      const float b0 = max_over_heads(head_live ? z0 : -INFINITY);
      const float b1 = max_over_heads(head_live ? z1 : -INFINITY);
      if (hd < 2) {
        const int tok = 16 * hd + t;
        const bool live = s < S && (int64_t)blk[u] * 32 + tok < n;
        out[s * 32 + tok] = live ? order_key(hd == 0 ? b0 : b1) : 0u;
      }
    }
  }
}

template <int BITS>
__global__ __launch_bounds__(256) void select_sample_score(Layout L, const uint8_t* __restrict__ kcache,
                                                           const uint16_t* __restrict__ q, NRes nr, SelectOut so) {
  sample_score_body<BITS>(L, kcache, q, nr.n[blockIdx.y / L.n_kv_heads], so.samples, so.m_samples, (int)blockIdx.x,
                          (int)blockIdx.y);
}

// 256 threads per row: small enough to find room on a chip that another stream's scan keeps full
__device__ __forceinline__ void sample_rank_body(const int64_t n, int32_t k, const uint32_t* __restrict__ samples,
                                                 const int m_samples, uint32_t* __restrict__ spec, const int row) {
  __shared__ uint32_t hist[4096];
  __shared__ uint32_t wsum[4];
  __shared__ uint32_t s_bin, s_rem, s_bin1;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int64_t want = n < k ? n : k;
  uint32_t* sp = spec + 4 * row;
  if (want <= 0) {
    if (tid == 0) { sp[0] = 0xffffffffu; sp[1] = 0; sp[2] = 0xffffffffu; }
    return;
  }
  const uint32_t* in = samples + (int64_t)row * m_samples;
  for (int i = tid; i < 4096; i += 256) hist[i] = 0;
  __syncthreads();
  for (int i0 = 0; i0 < m_samples; i0 += 8 * 256) {        // 8 loads in flight per thread
    uint32_t key[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) key[i] = in[i0 + i * 256 + tid];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (key[i] != 0) atomicAdd(&hist[key[i] >> 20], 1u);
  }
  __syncthreads();
  // exclusive prefix over the threads of `sum`, and the total
  auto scan256 = [&](uint32_t sum, uint32_t* total) {
    uint32_t inc = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t a = __shfl_up(inc, o);
      if (lane >= o) inc += a;
    }
    __syncthreads();                                        // earlier readers of wsum are done
    if (lane == 63) wsum[w] = inc;
    __syncthreads();
    uint32_t running = inc - sum, tot = 0;
    for (int x = 0; x < 4; ++x) { if (x < w) running += wsum[x]; tot += wsum[x]; }
    *total = tot;
    return running;
  };
  // bins from the top: thread tid owns bins 4095 - 16 tid - i
  uint32_t h[16], sum = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) { h[i] = hist[4095 - (16 * tid + i)]; sum += h[i]; }
  uint32_t m;                                               // sampled slots that exist
  uint32_t running = scan256(sum, &m);
  const float kappa = (float)want * (float)m / (float)n;
  const float root = 3.0f + sqrtf(9.0f + kappa);
  const uint32_t r = (uint32_t)ceilf(root * root);
  if (r >= m) {                                             // short rows: everything is a candidate
    if (tid == 0) { sp[0] = 0; sp[1] = 0; sp[2] = 0; }
    return;
  }
  // a second, deeper threshold for the case that the first one turns out too high: the lower bound of the 12-bit
  // bin that holds the 8r-th largest sample (0 if there is no such sample).  The scan counts the slots at or
  // above it, so that the selection knows whether a second scan with it is enough.
  const uint32_t r1 = 8 * r;
  if (tid == 0) sp[2] = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    if (running < r && r <= running + h[i]) { s_bin = 4095 - (16 * tid + i); s_rem = r - running; }
    if (running < r1 && r1 <= running + h[i]) s_bin1 = 4095 - (16 * tid + i);
    running += h[i];
  }
  __syncthreads();
  if (tid == 0 && r1 < m) sp[2] = s_bin1 << 20;
  const uint32_t bin = s_bin, rem = s_rem;
  for (int i = tid; i < 1024; i += 256) hist[i] = 0;
  __syncthreads();
  for (int i0 = 0; i0 < m_samples; i0 += 8 * 256) {
    uint32_t key[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) key[i] = in[i0 + i * 256 + tid];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (key[i] != 0 && (key[i] >> 20) == bin) atomicAdd(&hist[(key[i] >> 10) & 1023u], 1u);
  }
  __syncthreads();
  uint32_t g[4];
  sum = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) { g[i] = hist[1023 - (4 * tid + i)]; sum += g[i]; }
  uint32_t unused;
  running = scan256(sum, &unused);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (running < rem && rem <= running + g[i]) {
      sp[0] = (bin << 20) | ((uint32_t)(1023 - (4 * tid + i)) << 10);
      sp[1] = 0;
    }
    running += g[i];
  }
}

__global__ __launch_bounds__(256) void select_sample_rank(Layout L, NRes nr, int32_t k, SelectOut so) {
  sample_rank_body(nr.n[blockIdx.x / L.n_kv_heads], k, so.samples, so.m_samples, so.spec, (int)blockIdx.x);
}

// The two small jobs of a layer that precede its selecting scan in a decode step, as one launch: workgroup
// (0, row) turns the row's samples into its threshold (lengths `nr_after`, the new token included), workgroup
// (1, row) quantises and appends the step's key (lengths `nr_before`).
template <int BITS>
__global__ __launch_bounds__(256) void select_rank_append(Layout L, NRes nr_before, NRes nr_after, int32_t k,
                                                          SelectOut so, uint8_t* __restrict__ kcache,
                                                          const uint16_t* __restrict__ k_new,
                                                          float* __restrict__ acc, int32_t* __restrict__ pos,
                                                          NRes vrow0) {
  const int seq = blockIdx.y / L.n_kv_heads;
  if (blockIdx.x == 0) sample_rank_body(nr_after.n[seq], k, so.samples, so.m_samples, so.spec, (int)blockIdx.y);
  else quantize_body<BITS>(L, kcache, k_new, 1, nr_before.n[seq], acc, pos, vrow0.n[seq], 0, (int)blockIdx.y);
}

// One launch per layer for a decode step: the selecting scan of layer l with, as extra workgroups in front of its
// own, the sampling of layer l + 2 (m / 512 workgroups per row), the threshold of layer l + 1 from the samples that
// the previous launch took (one workgroup per row) and the append of layer l + 1's key (one workgroup per row).
// The roles touch different layers and do not depend on each other; what one launch writes the next one reads.
struct StepJob {
  // layer l + 1: threshold + append (a_on = 0: none)
  uint8_t* a_kcache;
  const uint16_t* a_k_new;
  float* a_acc;
  int32_t* a_pos;
  const uint32_t* a_samples;
  uint32_t* a_spec;
  int64_t a_vrow0;
  int32_t a_k, a_m, a_on;
  // layer l + 2: sampling (b_m = 0: none)
  const uint8_t* b_kcache;
  const uint16_t* b_q;
  uint32_t* b_samples;
  int32_t b_m;
  NRes a_nr, b_nr;            // lengths before the layers' own appends
};
template <int BITS, int U>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4))) void score_select_step_kernel(Layout L, const uint8_t* __restrict__ kcache,
                                                                const uint16_t* __restrict__ q, NRes nr, int bpw,
                                                                uint64_t* __restrict__ stamps, SelectOut so, StepJob j) {
  const int nsb = j.b_m / kSamplePerWg;
  const int extra = nsb + (j.a_on ? 2 : 0);
  const int bx = blockIdx.x, row = blockIdx.y;
  if (bx < nsb) {
    sample_score_body<BITS>(L, j.b_kcache, j.b_q, j.b_nr.n[row / L.n_kv_heads], j.b_samples, j.b_m, bx, row);
    return;
  }
  if (bx < extra) {
    const int64_t n_before = j.a_nr.n[row / L.n_kv_heads];
    if (bx == nsb) sample_rank_body(n_before + 1, j.a_k, j.a_samples, j.a_m, j.a_spec, row);
    else quantize_body<BITS>(L, j.a_kcache, j.a_k_new, 1, n_before, j.a_acc, j.a_pos, j.a_vrow0, 0, row);
    return;
  }
  score_body<BITS, false, U, false, true>(L, kcache, q, nr.n[row / L.n_kv_heads], bpw, nullptr, nullptr, stamps, 0.f,
                                          nullptr, so, bx - extra, (int)gridDim.x - extra, row);
}

// Two layers in one launch (the step driver's paired form): grid.y = 2 x rows, the upper half belongs to the
// second layer.  Each side is a complete score_select_step_kernel job with its own lengths, chunk count and
// extra workgroups; a workgroup beyond its side's needs returns at once.  One launch instead of two halves
// the pauses of the key stream between launches and the launch's tail is paid once for two layers.
struct StepSide {
  const uint8_t* kcache;          // the layer whose cache is scanned
  const uint16_t* q;
  uint64_t* stamps;
  SelectOut so;
  int32_t bpw, chunks;            // blocks per wave and chunks per row of this side's scan
  NRes32 nr;
  // threshold + append of the layer two on (a_on = 0: none)
  uint8_t* a_kcache;
  const uint16_t* a_k_new;
  float* a_acc;
  int32_t* a_pos;
  const uint32_t* a_samples;
  uint32_t* a_spec;
  int64_t a_vrow0;
  int32_t a_k, a_m, a_on;
  // sampling of the layer four on (b_m = 0: none)
  const uint8_t* b_kcache;
  const uint16_t* b_q;
  uint32_t* b_samples;
  int32_t b_m;
  NRes32 a_nr, b_nr;              // lengths before those layers' own appends
};

template <int BITS, int U>
__device__ __forceinline__ void step_side(const Layout& L, const StepSide& s, const int row) {
  const int nsb = s.b_m / kSamplePerWg;
  const int extra = nsb + (s.a_on ? 2 : 0);
  const int bx = blockIdx.x;
  const int seq = row / L.n_kv_heads;
  if (bx < nsb) {
    sample_score_body<BITS>(L, s.b_kcache, s.b_q, s.b_nr.n[seq], s.b_samples, s.b_m, bx, row);
    return;
  }
  if (bx < extra) {
    const int64_t n_before = s.a_nr.n[seq];
    if (bx == nsb) sample_rank_body(n_before + 1, s.a_k, s.a_samples, s.a_m, s.a_spec, row);
    else quantize_body<BITS>(L, s.a_kcache, s.a_k_new, 1, n_before, s.a_acc, s.a_pos, s.a_vrow0, 0, row);
    return;
  }
  if (bx - extra >= s.chunks) return;
  score_body<BITS, false, U, false, true>(L, s.kcache, s.q, s.nr.n[seq], s.bpw, nullptr, nullptr, s.stamps, 0.f, nullptr,
                                          s.so, bx - extra, s.chunks, row);
}

template <int BITS, int U>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4))) void score_select_pair_kernel(Layout L, StepSide s0, StepSide s1) {
  if ((int)blockIdx.y < L.rows) step_side<BITS, U>(L, s0, (int)blockIdx.y);
  else step_side<BITS, U>(L, s1, (int)blockIdx.y - L.rows);
}

// The start of a decode step in two launches instead of one per layer and job: the sampling of the first layers
// of every chain (up to four layers), then the threshold + append of the chains' first layers (up to two).
struct BeginSample {
  const uint8_t* kcache;
  const uint16_t* q;
  uint32_t* samples;
  int32_t m;
  NRes32 nr;
};
struct BeginSampleArgs { BeginSample s[4]; int32_t n; };
template <int BITS>
__global__ __launch_bounds__(256) void select_begin_samples(Layout L, BeginSampleArgs a) {
  const int side = (int)blockIdx.y / L.rows, row = (int)blockIdx.y % L.rows;
  const BeginSample& s = a.s[side];
  if ((int)blockIdx.x >= s.m / kSamplePerWg) return;
  sample_score_body<BITS>(L, s.kcache, s.q, s.nr.n[row / L.n_kv_heads], s.samples, s.m, (int)blockIdx.x, row);
}
struct BeginRank {
  uint8_t* kcache;
  const uint16_t* k_new;
  float* acc;
  int32_t* pos;
  const uint32_t* samples;
  uint32_t* spec;
  int64_t vrow0;
  int32_t k, m;
  NRes32 nr_before;
};
struct BeginRankArgs { BeginRank s[2]; int32_t n; };
template <int BITS>
__global__ __launch_bounds__(256) void select_begin_rank_append(Layout L, BeginRankArgs a) {
  const int side = (int)blockIdx.y / L.rows, row = (int)blockIdx.y % L.rows;
  const BeginRank& s = a.s[side];
  const int64_t n_before = s.nr_before.n[row / L.n_kv_heads];
  if (blockIdx.x == 0) sample_rank_body(n_before + 1, s.k, s.samples, s.m, s.spec, row);
  else quantize_body<BITS>(L, s.kcache, s.k_new, 1, n_before, s.acc, s.pos, s.vrow0, 0, row);
}

int32_t launch_select_begin_samples(const Layout& L, int n, const void* const kcache[], const void* const q[],
                                    const NRes nr[], const SelectOut so[], hipStream_t st) {
  if (n < 1 || n > 4) return HCA_ERR_BAD_ARG;
  BeginSampleArgs a;
  a.n = n;
  unsigned gx = 1;
  for (int i = 0; i < n; ++i) {
    a.s[i].kcache = (const uint8_t*)kcache[i];
    a.s[i].q = (const uint16_t*)q[i];
    a.s[i].samples = so[i].samples;
    a.s[i].m = so[i].m_samples;
    for (int b = 0; b < kMaxBatch; ++b) a.s[i].nr.n[b] = (int32_t)nr[i].n[b];
    if ((unsigned)(a.s[i].m / kSamplePerWg) > gx) gx = (unsigned)(a.s[i].m / kSamplePerWg);
  }
  for (int i = n; i < 4; ++i) a.s[i] = a.s[0];
  dim3 grid(gx, (unsigned)(n * L.rows));
  if (L.bits == 4) select_begin_samples<4><<<grid, 256, 0, st>>>(L, a);
  else select_begin_samples<2><<<grid, 256, 0, st>>>(L, a);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

int32_t launch_select_begin_rank_append(const Layout& L, int n, void* const kcache[], const void* const k_new[],
                                        const NRes nr_before[], float* const acc[], int32_t* const pos[],
                                        int64_t vrow0, int32_t k, const SelectOut so[], hipStream_t st) {
  if (n < 1 || n > 2) return HCA_ERR_BAD_ARG;
  BeginRankArgs a;
  a.n = n;
  for (int i = 0; i < n; ++i) {
    a.s[i].kcache = (uint8_t*)kcache[i];
    a.s[i].k_new = (const uint16_t*)k_new[i];
    a.s[i].acc = acc[i];
    a.s[i].pos = pos[i];
    a.s[i].samples = so[i].samples;
    a.s[i].spec = so[i].spec;
    a.s[i].vrow0 = vrow0;
    a.s[i].k = k;
    a.s[i].m = so[i].m_samples;
    for (int b = 0; b < kMaxBatch; ++b) a.s[i].nr_before.n[b] = (int32_t)nr_before[i].n[b];
  }
  for (int i = n; i < 2; ++i) a.s[i] = a.s[0];
  dim3 grid(2, (unsigned)(n * L.rows));
  if (L.bits == 4) select_begin_rank_append<4><<<grid, 256, 0, st>>>(L, a);
  else select_begin_rank_append<2><<<grid, 256, 0, st>>>(L, a);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

// Slots to sample per row.  More samples give a tighter threshold: with m samples the scan lets through about
// n r / m pairs per row, r as in the comment above.  The smallest of 8192 .. 65536 that keeps that estimate within
// what the selection holds in LDS (16384 pairs, less a margin for the spread of the count).
int select_sample_count(int64_t nmax, int32_t k) {
  int m = 8192;
  for (; m < 65536; m *= 2) {
    const double want = (double)(k < nmax ? k : nmax);
    const double kappa = want * m / (double)(nmax > 0 ? nmax : 1);
    const double root = 3.0 + sqrt(9.0 + kappa);
    const double r = root * root;
    if (r >= m || (double)nmax * r / m <= 14336.0) break;
  }
  return m;
}

int select_scan_bpw(const Layout& L, int64_t nmax) {
  const int64_t nblocks = (nmax + L.tpb - 1) / L.tpb;
  const int64_t total = nblocks * L.rows;
  int64_t bpw = total / (256 * 4 * 16);
  if (bpw < 4) bpw = 4;
  const int64_t bpw_max = L.bits == 4 ? 16 : 32;
  if (bpw > bpw_max) bpw = bpw_max;
  const int64_t need = (nblocks + 4 * kSelectMaxChunks - 1) / (4 * kSelectMaxChunks);   // chunks per row <= 1024
  if (bpw < need) bpw = (need + 7) / 8 * 8;
  if (4 * bpw * L.tpb * (int64_t)sizeof(uint2) > 64 * 1024) return 0;                     // wave lists no longer fit
  return (int)bpw;
}

int32_t launch_select_sample_scores(const Layout& L, const void* kcache, const void* q, const NRes& nr,
                                    const SelectOut& so, hipStream_t st) {
  const uint8_t* kc = (const uint8_t*)kcache;
  const uint16_t* qq = (const uint16_t*)q;
  dim3 grid((unsigned)(so.m_samples / kSamplePerWg), (unsigned)L.rows);
  if (L.bits == 4) select_sample_score<4><<<grid, 256, 0, st>>>(L, kc, qq, nr, so);
  else select_sample_score<2><<<grid, 256, 0, st>>>(L, kc, qq, nr, so);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

int32_t launch_select_sample(const Layout& L, const void* kcache, const void* q, const NRes& nr, int32_t k,
                             const SelectOut& so, hipStream_t st) {
  const int32_t rc = launch_select_sample_scores(L, kcache, q, nr, so, st);
  if (rc != HCA_OK) return rc;
  select_sample_rank<<<L.rows, 256, 0, st>>>(L, nr, k, so);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

int32_t launch_select_rank_append(const Layout& L, void* kcache, const void* k_new, const NRes& nr_before, float* acc,
                                  int32_t* pos, const NRes& vrow0, int32_t k, const SelectOut& so, hipStream_t st) {
  NRes after = nr_before;
  for (int b = 0; b < L.batch; ++b) after.n[b] += 1;
  dim3 grid(2, (unsigned)L.rows);
  if (L.bits == 4)
    select_rank_append<4><<<grid, 256, 0, st>>>(L, nr_before, after, k, so, (uint8_t*)kcache, (const uint16_t*)k_new, acc,
                                                pos, vrow0);
  else
    select_rank_append<2><<<grid, 256, 0, st>>>(L, nr_before, after, k, so, (uint8_t*)kcache, (const uint16_t*)k_new, acc,
                                                pos, vrow0);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

int32_t launch_select_step(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax,
                           const SelectOut& so, hipStream_t st, uint64_t* stamps, const SelectStepNext& nx) {
  if (nmax == 0) return HCA_ERR_BAD_ARG;
  const int bpw = select_scan_bpw(L, nmax);
  if (bpw == 0) return HCA_ERR_CAPACITY;
  const int64_t nblocks = (nmax + L.tpb - 1) / L.tpb;
  StepJob j;
  j.a_kcache = (uint8_t*)nx.a_kcache;
  j.a_k_new = (const uint16_t*)nx.a_k_new;
  j.a_acc = nx.a_acc;
  j.a_pos = nx.a_pos;
  j.a_samples = nx.a_so.samples;
  j.a_spec = nx.a_so.spec;
  j.a_vrow0 = nx.a_vrow0;
  j.a_k = nx.k;
  j.a_m = nx.a_so.m_samples;
  j.a_on = nx.a_kcache != nullptr;
  j.b_kcache = (const uint8_t*)nx.b_kcache;
  j.b_q = (const uint16_t*)nx.b_q;
  j.b_samples = nx.b_so.samples;
  j.b_m = nx.b_kcache != nullptr ? nx.b_so.m_samples : 0;
  j.a_nr = nx.a_nr;
  j.b_nr = nx.b_nr;
  const unsigned extra = (unsigned)(j.b_m / kSamplePerWg) + (j.a_on ? 2u : 0u);
  dim3 grid((unsigned)((nblocks + 4 * bpw - 1) / (4 * bpw)) + extra, (unsigned)L.rows);
  const size_t lds = (size_t)4 * bpw * L.tpb * sizeof(uint2);
  if (L.bits == 4)
    score_select_step_kernel<4, 8><<<grid, 256, lds, st>>>(L, (const uint8_t*)kcache, (const uint16_t*)q, nr, bpw, stamps,
                                                           so, j);
  else
    score_select_step_kernel<2, 8><<<grid, 256, lds, st>>>(L, (const uint8_t*)kcache, (const uint16_t*)q, nr, bpw, stamps,
                                                           so, j);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

static int32_t fill_side(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax,
                         const SelectOut& so, uint64_t* stamps, const SelectStepNext& nx, StepSide* s, unsigned* gx,
                         size_t* lds) {
  if (nmax == 0) return HCA_ERR_BAD_ARG;
  const int bpw = select_scan_bpw(L, nmax);
  if (bpw == 0) return HCA_ERR_CAPACITY;
  const int64_t nblocks = (nmax + L.tpb - 1) / L.tpb;
  s->kcache = (const uint8_t*)kcache;
  s->q = (const uint16_t*)q;
  s->stamps = stamps;
  s->so = so;
  s->bpw = bpw;
  s->chunks = (int32_t)((nblocks + 4 * bpw - 1) / (4 * bpw));
  for (int b = 0; b < kMaxBatch; ++b) {
    s->nr.n[b] = (int32_t)nr.n[b];
    s->a_nr.n[b] = (int32_t)nx.a_nr.n[b];
    s->b_nr.n[b] = (int32_t)nx.b_nr.n[b];
  }
  s->a_kcache = (uint8_t*)nx.a_kcache;
  s->a_k_new = (const uint16_t*)nx.a_k_new;
  s->a_acc = nx.a_acc;
  s->a_pos = nx.a_pos;
  s->a_samples = nx.a_so.samples;
  s->a_spec = nx.a_so.spec;
  s->a_vrow0 = nx.a_vrow0;
  s->a_k = nx.k;
  s->a_m = nx.a_so.m_samples;
  s->a_on = nx.a_kcache != nullptr;
  s->b_kcache = (const uint8_t*)nx.b_kcache;
  s->b_q = (const uint16_t*)nx.b_q;
  s->b_samples = nx.b_so.samples;
  s->b_m = nx.b_kcache != nullptr ? nx.b_so.m_samples : 0;
  const unsigned g = (unsigned)s->chunks + (unsigned)(s->b_m / kSamplePerWg) + (s->a_on ? 2u : 0u);
  if (g > *gx) *gx = g;
  const size_t l = (size_t)4 * bpw * L.tpb * sizeof(uint2);
  if (l > *lds) *lds = l;
  return HCA_OK;
}

// The selecting scans of two layers (and what each carries for the layers behind it) as one launch.
// `done` (optional): an event that completes with this launch.  It is bound to the dispatch itself
// (hipExtLaunchKernelGGL's stop event) instead of being recorded behind it: a recorded event is a packet of its
// own on the stream, and the next scan launch waits ~8 us for it.
int32_t launch_select_step_pair(const Layout& L, const void* const kcache[2], const void* const q[2], const NRes nr[2],
                                const int64_t nmax[2], const SelectOut so[2], uint64_t* const stamps[2],
                                const SelectStepNext nx[2], hipStream_t st, hipEvent_t done) {
  StepSide s0, s1;
  unsigned gx = 0;
  size_t lds = 0;
  int32_t rc = fill_side(L, kcache[0], q[0], nr[0], nmax[0], so[0], stamps[0], nx[0], &s0, &gx, &lds);
  if (rc != HCA_OK) return rc;
  rc = fill_side(L, kcache[1], q[1], nr[1], nmax[1], so[1], stamps[1], nx[1], &s1, &gx, &lds);
  if (rc != HCA_OK) return rc;
  dim3 grid(gx, (unsigned)(2 * L.rows));
  if (done != nullptr) {
    if (L.bits == 4)
      hipExtLaunchKernelGGL((score_select_pair_kernel<4, 8>), grid, dim3(256), (uint32_t)lds, st, nullptr, done, 0, L, s0, s1);
    else
      hipExtLaunchKernelGGL((score_select_pair_kernel<2, 8>), grid, dim3(256), (uint32_t)lds, st, nullptr, done, 0, L, s0, s1);
  } else {
    if (L.bits == 4) score_select_pair_kernel<4, 8><<<grid, 256, lds, st>>>(L, s0, s1);
    else score_select_pair_kernel<2, 8><<<grid, 256, lds, st>>>(L, s0, s1);
  }
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

int32_t launch_select_rescan_pair(const Layout& L, const void* const kcache[2], const void* const q[2], const NRes nr[2],
                                  const int64_t nmax[2], const SelectOut so[2], hipStream_t st) {
  RescanSide rs[2];
  unsigned gx = 1;
  size_t lds = 0;
  for (int i = 0; i < 2; ++i) {
    const int bpw = select_scan_bpw(L, nmax[i]);
    if (bpw == 0) return HCA_ERR_CAPACITY;
    const int64_t nblocks = (nmax[i] + L.tpb - 1) / L.tpb;
    rs[i].kcache = (const uint8_t*)kcache[i];
    rs[i].q = (const uint16_t*)q[i];
    rs[i].so = so[i];
    rs[i].bpw = bpw;
    rs[i].nchunks = (int32_t)((nblocks + 4 * bpw - 1) / (4 * bpw));
    for (int b = 0; b < kMaxBatch; ++b) rs[i].nr.n[b] = (int32_t)nr[i].n[b];
    if ((unsigned)rs[i].nchunks > gx) gx = (unsigned)rs[i].nchunks;
    const size_t l = (size_t)4 * bpw * L.tpb * sizeof(uint2);
    if (l > lds) lds = l;
  }
  // 16 workgroups per row, not the 256 of the per-call path: nearly always no row failed and every workgroup
  // returns at once, but beside a running scan 4096 of them take a slot each first (0.2 ms per step at config 4)
  dim3 grid(gx < 16 ? gx : 16, (unsigned)(2 * L.rows));
  if (L.bits == 4) score_failed_rows_pair_kernel<4, 8><<<grid, 256, lds, st>>>(L, rs[0], rs[1]);
  else score_failed_rows_pair_kernel<2, 8><<<grid, 256, lds, st>>>(L, rs[0], rs[1]);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

int32_t launch_select_scan(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax,
                           const SelectOut& so, bool only_failed, hipStream_t st, uint64_t* stamps) {
  if (nmax == 0) return HCA_OK;
  const int bpw = select_scan_bpw(L, nmax);
  if (bpw == 0) return HCA_ERR_CAPACITY;
  const int64_t nblocks = (nmax + L.tpb - 1) / L.tpb;
  dim3 grid((unsigned)((nblocks + 4 * bpw - 1) / (4 * bpw)), (unsigned)L.rows);
  const size_t lds = (size_t)4 * bpw * L.tpb * sizeof(uint2);
  const uint8_t* kc = (const uint8_t*)kcache;
  const uint16_t* qq = (const uint16_t*)q;
  if (only_failed) {
    dim3 small(grid.x < 256 ? grid.x : 256, (unsigned)L.rows);
    if (L.bits == 4) score_failed_rows_kernel<4, 8><<<small, 256, lds, st>>>(L, kc, qq, nr, bpw, (int)grid.x, so);
    else score_failed_rows_kernel<2, 8><<<small, 256, lds, st>>>(L, kc, qq, nr, bpw, (int)grid.x, so);
  } else if (L.bits == 4) {
    score_select_kernel<4, 8><<<grid, 256, lds, st>>>(L, kc, qq, nr, bpw, stamps, so);
  } else {
    score_select_kernel<2, 8><<<grid, 256, lds, st>>>(L, kc, qq, nr, bpw, stamps, so);
  }
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

// number of (start, end) stamp pairs a scan launch over nmax tokens writes at most
int64_t score_stamp_pairs(const Layout& L, int64_t nmax) {
  const int64_t nblocks = (nmax + L.tpb - 1) / L.tpb;
  return (nblocks / kScoreBpwMin + 4) * L.rows;   // >= grid.x * 4 waves * rows for any blocks-per-wave >= kScoreBpwMin
}

// float2 pairs a scan launch with LSE leaves per row: 4 heads x (waves of the row), for any blocks-per-wave >= 4
size_t score_workspace_bytes(const Layout& L) {
  return (size_t)L.rows * 4 * (size_t)(L.nblk / 4 + 8) * sizeof(float2);
}

int32_t launch_score(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax,
                     float* sel, float* z_opt, hipStream_t st, uint64_t* stamps, const Tuning* tune) {
  if (nmax == 0) return HCA_OK;
  const int64_t nblocks = (nmax + L.tpb - 1) / L.tpb;
  // aim at ~16 waves per SIMD over the whole chip when the cache is large, >= 4 blocks per wave
  const int64_t total = nblocks * L.rows;
  const Tuning& tn = tune != nullptr ? *tune : tuning();
  int64_t bpw = total / (256 * 4 * 16);
  if (bpw < 4) bpw = 4;
  // measured best on MI355X: 4-bit codes 8 blocks ahead, 16 per wave; 2-bit codes (two tiles per block,
  // more registers) 4 ahead, 32 per wave
  const int64_t bpw_max = L.bits == 4 ? 16 : 32;
  if (bpw > bpw_max) bpw = bpw_max;
  if (tn.score_bpw > 0) bpw = tn.score_bpw;
  if (bpw < kScoreBpwMin) bpw = kScoreBpwMin;
  if (bpw > kScoreBpwMax) bpw = kScoreBpwMax;
  const int depth = tn.score_depth > 0 ? tn.score_depth : 8;
  dim3 grid((unsigned)((nblocks + 4 * bpw - 1) / (4 * bpw)), (unsigned)L.rows);
  // every wave of the launch owns one stamp pair: the caller's buffer holds score_stamp_pairs() of them
  if (stamps != nullptr && (int64_t)grid.x * 4 * L.rows > score_stamp_pairs(L, nmax)) return HCA_ERR_CAPACITY;
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
  if (tn.score_bpw >= kScoreBpwMin) bpw = tn.score_bpw;
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
