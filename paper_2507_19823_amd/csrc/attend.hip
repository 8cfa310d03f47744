// Step 3b: gather of the selected value rows (pinned host memory and / or an HBM slice) and the
// softmax-weighted sum over the selected set (Eq. 5), plus the accumulated-score update.
#include "hca_internal.h"

namespace hca {

constexpr int kChunk = kAttendChunk;  // selected tokens per workgroup of the partial kernel

struct AttendWs {
  uint16_t* vstage;  // [rows][k][128] fp16
  float* logit;      // [rows][4][k]
  float* pmz;        // [rows][nsplit][4][2]  (max, sum) per chunk
  float* py;         // [rows][nsplit][4][128]
};

static int nsplit_of(int64_t k) { return (int)((k + kChunk - 1) / kChunk); }

size_t attend_workspace_bytes(const Layout& L, int64_t k) {
  const int64_t ns = nsplit_of(k);
  size_t b = 0;
  b += align_up((int64_t)L.rows * k * kHeadDim * 2, 256);
  b += align_up((int64_t)L.rows * 4 * k * 4, 256);
  b += align_up((int64_t)L.rows * ns * 4 * 2 * 4, 256);
  b += align_up((int64_t)L.rows * ns * 4 * kHeadDim * 4, 256);
  return b;
}

static void carve(AttendWs* a, void* ws, const Layout& L, int64_t k) {
  const int64_t ns = nsplit_of(k);
  uint8_t* w = (uint8_t*)ws;
  a->vstage = (uint16_t*)w; w += align_up((int64_t)L.rows * k * kHeadDim * 2, 256);
  a->logit = (float*)w;     w += align_up((int64_t)L.rows * 4 * k * 4, 256);
  a->pmz = (float*)w;       w += align_up((int64_t)L.rows * ns * 4 * 2 * 4, 256);
  a->py = (float*)w;
}

// 16 threads move one 256-byte value row; rows below n_host_rows are read straight from
// pinned host memory over the host link (zero-copy), the others from the HBM slice.  The grid
// is deliberately small and persistent: the host link saturates with a few hundred KiB in
// flight, and more outstanding host reads than that only clog the memory pipeline for the
// HBM-bound kernels that run beside the gather.
template <int UNROLL>
__global__ __launch_bounds__(256) void gather_values(const int32_t* __restrict__ idx, const int32_t* __restrict__ count,
                                                     int32_t k, const int32_t* __restrict__ pos, int64_t cap,
                                                     const uint4* __restrict__ v_host, int64_t host_stride,
                                                     int64_t n_host_rows, const uint4* __restrict__ v_hbm,
                                                     int64_t hbm_stride, uint4* __restrict__ vstage,
                                                     int wgs, uint64_t* __restrict__ stamps, int first,
                                                     uint32_t* __restrict__ gpu_seq, uint32_t seq) {
  const int row = blockIdx.y, wg = blockIdx.x;
  // hybrid value side: the kernel before this one on the stream left the host's inputs in pinned memory; a
  // kernel starts only when its predecessor's stores are visible, so the first thing this one does is tell the host
  if (gpu_seq != nullptr && row == 0 && wg == 0 && threadIdx.x == 0)
    __hip_atomic_store(gpu_seq, seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  // optional profiling: every workgroup leaves its start and end time (constant-rate wall clock)
  uint64_t* stamp = stamps ? stamps + ((int64_t)row * wgs + wg) * 2 : nullptr;
  if (stamp && threadIdx.x == 0) stamp[0] = wall_clock64();
  const int cnt = count[row];
  const int part = threadIdx.x & 15;
  const int64_t step = (int64_t)wgs * 16;                 // value rows per sweep of the row's workgroups
  // entries below `first` are not fetched (their values are summed where they live, on the host)
  for (int64_t i0 = (int64_t)first + (int64_t)wg * 16 + (threadIdx.x >> 4); i0 < cnt; i0 += step * UNROLL) {
    uint4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int64_t i = i0 + u * step;
      if (i < cnt) {
        const int32_t slot = idx[(int64_t)row * k + i];
        const int64_t vr = pos[(int64_t)row * cap + slot];
        const uint4* src = (vr < n_host_rows) ? v_host + ((int64_t)row * host_stride + vr) * 16
                                              : v_hbm + ((int64_t)row * hbm_stride + (vr - n_host_rows)) * 16;
        // read-once rows, write-once staging: non-temporal both ways, so that neither side displaces or
        // queues behind what the HBM-bound kernels beside the gather keep in the caches
        const v4i t4 = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(src + part));
        v[u] = uint4{(uint32_t)t4.x, (uint32_t)t4.y, (uint32_t)t4.z, (uint32_t)t4.w};
      }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int64_t i = i0 + u * step;
      if (i < cnt) {
        const v4i t4 = {(int)v[u].x, (int)v[u].y, (int)v[u].z, (int)v[u].w};
        __builtin_nontemporal_store(t4, reinterpret_cast<v4i*>(vstage + ((int64_t)row * k + i) * 16 + part));
      }
    }
  }
  if (stamp) {
    __syncthreads();
    if (threadIdx.x == 0) stamp[1] = wall_clock64();
  }
}

// Shared memory of one chunk (256 selected tokens, up to 4 query heads) of the partial kernels.
struct PartialShared {
  float lg[4][kChunk];          // logits, then exp(logit - chunk max)
  float red[4][4][kHeadDim];
  float hm[4], hz[4];
};

// Writes the neutral partial of an empty chunk.
__device__ __forceinline__ void partial_empty(float* pmz, float* py) {
  if (threadIdx.x < 4) { pmz[2 * threadIdx.x] = -INFINITY; pmz[2 * threadIdx.x + 1] = 0.f; }
  for (int c = threadIdx.x; c < 4 * kHeadDim; c += 256) py[c] = 0.f;
}

// Steps 2 and 3 of a chunk, after its logits sit in ps.lg (and a __syncthreads()): per-head chunk
// max / exponentials / sum, then the weighted sum of the staged value rows.
template <bool VALUES = true>
__device__ __forceinline__ void partial_softmax_sum(PartialShared& ps, const AttendWs& a, int row, int i0, int nvalid,
                                                    int32_t k, float* pmz, float* py) {
  auto& lg = ps.lg;
  auto& red = ps.red;
  auto& hm = ps.hm;
  auto& hz = ps.hz;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  // 2. per head (wave w = head w): chunk max, exponentials, chunk sum
  {
    float m = -INFINITY;
    for (int i = lane; i < nvalid; i += 64) m = fmaxf(m, lg[w][i]);
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    float z = 0.f;
    for (int i = lane; i < nvalid; i += 64) {
      const float l = lg[w][i];
      a.logit[((int64_t)row * 4 + w) * k + i0 + i] = l;
      const float p = expf(l - m);
      lg[w][i] = p;
      z += p;
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) z += __shfl_xor(z, o);
    if (lane == 0) { hm[w] = m; hz[w] = z; }
  }
  __syncthreads();
  if constexpr (!VALUES) {   // weights only: the chunk's (max, sum) pairs and the stored logits are all that is needed
    if (threadIdx.x < 4) { pmz[2 * threadIdx.x] = hm[threadIdx.x]; pmz[2 * threadIdx.x + 1] = hz[threadIdx.x]; }
    return;
  }

  // 3. weighted value sum.  Wave w owns tokens [64w, 64w+64) of the chunk; one load instruction
  //    fetches 4 staged rows (lane>>4 picks the row, lane&15 its 16-byte part) and 8 of them are
  //    issued before the first is used.
  float acc[4][8];
#pragma unroll
  for (int h = 0; h < 4; ++h)
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[h][c] = 0.f;
  const int part = lane & 15, sub = lane >> 4;
  const uint4* vs = reinterpret_cast<const uint4*>(a.vstage) + ((int64_t)row * k + i0) * 16 + part;
  for (int it = 0; it < 16; it += 8) {
    uint4 rv[8];
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      const int i = 64 * w + 4 * (it + x) + sub;
      rv[x] = vs[(int64_t)(i < nvalid ? i : nvalid - 1) * 16];
    }
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      const int i = 64 * w + 4 * (it + x) + sub;
      if (i < nvalid) {
        const uint32_t wd[4] = {rv[x].x, rv[x].y, rv[x].z, rv[x].w};
        float v[8];
#pragma unroll
        for (int c = 0; c < 4; ++c) { v[2 * c] = h2f(wd[c] & 0xffffu); v[2 * c + 1] = h2f(wd[c] >> 16); }
#pragma unroll
        for (int h = 0; h < 4; ++h) {
          const float p = lg[h][i];
#pragma unroll
          for (int c = 0; c < 8; ++c) acc[h][c] = fmaf(p, v[c], acc[h][c]);
        }
      }
    }
  }
#pragma unroll
  for (int h = 0; h < 4; ++h)
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      float x = acc[h][c];
      x += __shfl_xor(x, 16);
      x += __shfl_xor(x, 32);
      acc[h][c] = x;
    }
  if (sub == 0) {
#pragma unroll
    for (int h = 0; h < 4; ++h)
#pragma unroll
      for (int c = 0; c < 8; ++c) red[w][h][8 * part + c] = acc[h][c];
  }
  __syncthreads();
  for (int c = threadIdx.x; c < 4 * kHeadDim; c += 256) {
    const int h = c >> 7, d = c & 127;
    py[c] = (red[0][h][d] + red[1][h][d]) + (red[2][h][d] + red[3][h][d]);
  }
  if (threadIdx.x < 4) { pmz[2 * threadIdx.x] = hm[threadIdx.x]; pmz[2 * threadIdx.x + 1] = hz[threadIdx.x]; }
}

template <int BITS, bool VALUES = true>
__device__ __forceinline__ bool attend_partial_body(PartialShared& ps, QShared& sh, const Layout& L,
                                                    const uint8_t* __restrict__ kcache, const uint16_t* __restrict__ q,
                                                    const int32_t* __restrict__ idx, const int32_t* __restrict__ count,
                                                    int32_t k, float sm_scale, const AttendWs& a, int nsplit,
                                                    const int split) {
  auto& lg = ps.lg;
  const int row = blockIdx.y;
  const int cnt = count[row];
  const int i0 = split * kChunk;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int t = lane & 15, j = lane >> 4;
  float* pmz = a.pmz + (((int64_t)row * nsplit + split) * 4) * 2;
  float* py = a.py + (((int64_t)row * nsplit + split) * 4) * kHeadDim;
  if (i0 >= cnt) {  // empty chunk: neutral partial
    partial_empty(pmz, py);
    return false;
  }
  const int nvalid = (cnt - i0 < kChunk) ? cnt - i0 : kChunk;
  load_query(q, row, L.gqa, L.group, &sh);
  QOperand<BITS> op;
  build_operand<BITS>(&sh, &op);
  const uint8_t* crow = kcache + (int64_t)row * L.codes_row_bytes();
  const uint8_t* mrow = kcache + L.meta_off + (int64_t)row * L.meta_row_bytes();
  const int32_t* ridx = idx + (int64_t)row * k;

  // 1. logits of the chunk: wave w scores tiles w, w+4, w+8, w+12 (16 selected tokens each).
  //    All slot numbers are fetched first, then all code / meta pieces, so that the wave has its
  //    whole share of the random reads in flight at once.
  {
    int64_t slot[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const int i = (w + 4 * x) * 16 + t;
      slot[x] = ridx[i0 + (i < nvalid ? i : nvalid - 1)];
    }
    uint4 wv[4], mv[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      if constexpr (BITS == 4) {
        const int64_t blk = slot[x] >> 4;
        const int tl = (int)(slot[x] & 15);
        wv[x] = *reinterpret_cast<const uint4*>(crow + blk * kBlockBytes + (tl + 16 * j) * 16);
        mv[x] = *reinterpret_cast<const uint4*>(mrow + blk * kMetaBytes + tl * 16);
      } else {
        const int64_t blk = slot[x] >> 5;
        const int u = (int)((slot[x] >> 4) & 1), tl = (int)(slot[x] & 15);
        const uint2 c = *reinterpret_cast<const uint2*>(crow + blk * kBlockBytes + (tl + 16 * j) * 16 + 8 * u);
        const uint2 m = *reinterpret_cast<const uint2*>(mrow + blk * kMetaBytes + (16 * u + tl) * 8);
        wv[x] = uint4{c.x, c.y, 0, 0};
        mv[x] = uint4{m.x, m.y, 0, 0};
      }
    }
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      float zv;
      if constexpr (BITS == 4) zv = score_block4(op, wv[x], mv[x]);
      else zv = score_tile2(op, wv[x].x, wv[x].y, uint2{mv[x].x, mv[x].y});
      // lane (t, hd = j) holds z~ of head j for selected token (w + 4x)*16 + t
      lg[j][(w + 4 * x) * 16 + t] = zv * sm_scale;
    }
  }
  __syncthreads();

  partial_softmax_sum<VALUES>(ps, a, row, i0, nvalid, k, pmz, py);
  return true;
}

// split0: the first chunk of the launch (chunks below it belong to the host share)
template <int BITS, bool VALUES = true>
__global__ __launch_bounds__(256) void attend_partial(Layout L, const uint8_t* __restrict__ kcache,
                                                      const uint16_t* __restrict__ q, const int32_t* __restrict__ idx,
                                                      const int32_t* __restrict__ count, int32_t k, float sm_scale,
                                                      AttendWs a, int nsplit, int split0) {
  __shared__ QShared sh;
  __shared__ PartialShared ps;
  attend_partial_body<BITS, VALUES>(ps, sh, L, kcache, q, idx, count, k, sm_scale, a, nsplit, (int)blockIdx.x + split0);
}

// The chunks of the host share: logits, chunk (max, sum) and stored logits as for any chunk (the merge and the
// accumulated scores need them), no value rows; instead every entry's exp(logit - chunk max) per head and its
// value-row number go to pinned host memory.  An entry whose value row is not in the host store (rows >=
// n_host_rows live in the HBM slice: the newest tokens) is summed here, into the chunk's device-side partial,
// and is handed to the host as "nothing to add".
template <int BITS>
__global__ __launch_bounds__(256) void attend_host_chunks(Layout L, const uint8_t* __restrict__ kcache,
                                                          const uint16_t* __restrict__ q, const int32_t* __restrict__ idx,
                                                          const int32_t* __restrict__ count, int32_t k,
                                                          const int32_t* __restrict__ pos, int64_t n_host_rows,
                                                          const uint16_t* __restrict__ v_hbm, int64_t hbm_stride,
                                                          float sm_scale, AttendWs a, int nsplit, HostShare hs) {
  __shared__ QShared sh;
  __shared__ PartialShared ps;
  __shared__ int32_t vr[kChunk];
  __shared__ int n_dev;
  const int row = blockIdx.y, split = blockIdx.x;
  const int tid = threadIdx.x;
  float* out_p = hs.p + ((int64_t)row * hs.chunks + split) * 4 * kChunk;
  int32_t* out_v = hs.vrow + ((int64_t)row * hs.chunks + split) * kChunk;
  float* py = a.py + (((int64_t)row * nsplit + split) * 4) * kHeadDim;
  if (tid == 0) n_dev = 0;
  const bool live_chunk = attend_partial_body<BITS, false>(ps, sh, L, kcache, q, idx, count, k, sm_scale, a, nsplit, split);
  if (!live_chunk) {                  // nothing selected here: partial_empty has written the neutral partial
    out_v[tid] = -1;
#pragma unroll
    for (int h = 0; h < 4; ++h) out_p[h * kChunk + tid] = 0.f;
    return;
  }
  // ps.lg now holds exp(logit - chunk max) of the chunk's live entries
  const int cnt = count[row];
  const int i0 = split * kChunk;
  const int nvalid = (cnt - i0 < kChunk) ? cnt - i0 : kChunk;
  int32_t r = -1;
  bool on_dev = false;
  if (tid < nvalid) {
    const int32_t slot = idx[(int64_t)row * k + i0 + tid];
    const int32_t v = pos[(int64_t)row * L.cap + slot];
    on_dev = v >= n_host_rows;
    r = on_dev ? -1 : v;
    vr[tid] = on_dev ? (int32_t)(v - n_host_rows) : -1;
    if (on_dev) atomicAdd(&n_dev, 1);
  } else {
    vr[tid] = -1;
  }
  out_v[tid] = r;
#pragma unroll
  for (int h = 0; h < 4; ++h) out_p[h * kChunk + tid] = (tid < nvalid && h < L.gqa) ? ps.lg[h][tid] : 0.f;
  __syncthreads();
  // device-side partial of the chunk: the entries that the host cannot reach (usually none)
  for (int c = tid; c < 4 * kHeadDim; c += 256) {
    const int h = c >> 7, d = c & 127;
    float s = 0.f;
    if (n_dev > 0 && h < L.gqa) {
      for (int i = 0; i < nvalid; ++i) {
        const int32_t x = vr[i];
        if (x >= 0) s = fmaf(ps.lg[h][i], h2f(v_hbm[((int64_t)row * hbm_stride + x) * kHeadDim + d]), s);
      }
    }
    py[c] = s;
  }
}

// Table entry of one (group, centroid): the G query heads of the KV head, adjacent in memory.
template <int G>
__device__ __forceinline__ void load_entry(const float* p, float (&e)[G]) {
  if constexpr (G == 4) {
    const float4 v = *reinterpret_cast<const float4*>(p);
    e[0] = v.x; e[1] = v.y; e[2] = v.z; e[3] = v.w;
  } else if constexpr (G == 2) {
    const float2 v = *reinterpret_cast<const float2*>(p);
    e[0] = v.x; e[1] = v.y;
  } else {
    e[0] = p[0];
  }
}

// Codebook form: the logit of a selected token is the sum over the groups of the table entries
// its indices select (Eq. 3), added exactly on the table's power-of-two grid (the exponents that the
// scan left behind the table in `lut`).  Thread i of the chunk owns selected token i0 + i.
template <int G, bool WIDE>
__global__ __launch_bounds__(256) void vq_attend_partial(int g, int c, int64_t cap, const uint8_t* __restrict__ pcache,
                                                         const float* __restrict__ lut, const int32_t* __restrict__ idx,
                                                         const int32_t* __restrict__ count, int32_t k, float sm_scale,
                                                         AttendWs a, int nsplit) {
  __shared__ PartialShared ps;
  const int row = blockIdx.y, split = blockIdx.x;
  const int cnt = count[row];
  const int i0 = split * kChunk;
  float* pmz = a.pmz + (((int64_t)row * nsplit + split) * 4) * 2;
  float* py = a.py + (((int64_t)row * nsplit + split) * 4) * kHeadDim;
  if (i0 >= cnt) {
    partial_empty(pmz, py);
    return;
  }
  const int nvalid = (cnt - i0 < kChunk) ? cnt - i0 : kChunk;
  {
    const int i = threadIdx.x;
    const int64_t slot = idx[(int64_t)row * k + i0 + (i < nvalid ? i : nvalid - 1)];
    const uint8_t* pr = pcache + ((int64_t)row * cap + slot) * g;                  // narrow form: the slot's record
    const uint16_t* pw = reinterpret_cast<const uint16_t*>(pcache);
    const int64_t tiles = vq_tiles(cap);
    const float* T = lut + (int64_t)row * g * c * G;
    const int32_t* sexp = reinterpret_cast<const int32_t*>(lut + (int64_t)gridDim.y * g * (c * G + 4)) + row * 4;
    int s[G], zi[G];
#pragma unroll
    for (int h = 0; h < G; ++h) { s[h] = sexp[h]; zi[h] = 0; }
    for (int i16 = 0; i16 < g; i16 += 16) {
      int64_t ent[16];                          // entry number in the table of this row
      if constexpr (WIDE) {                     // 16-bit indices, group-major tiles; table [group][centroid]
#pragma unroll
        for (int b = 0; b < 16; ++b) {
          const int code = (int)pw[vq_wide_at(g, tiles, row, slot, i16 + b)];
          ent[b] = (int64_t)(i16 + b) * c + code;
        }
      } else {                                  // byte indices, rotated by the slot number; table [centroid][group]
        const uint4 pv = *reinterpret_cast<const uint4*>(pr + i16);
        const uint32_t wd[4] = {pv.x, pv.y, pv.z, pv.w};
#pragma unroll
        for (int b = 0; b < 16; ++b)
          ent[b] = (int64_t)((wd[b >> 2] >> (8 * (b & 3))) & 255u) * g + vq_group_at(i16 + b, slot);
      }
      float e[16][G];
#pragma unroll
      for (int b = 0; b < 16; ++b)              // 16 independent table reads in flight
        load_entry<G>(T + ent[b] * G, e[b]);
#pragma unroll
      for (int b = 0; b < 16; ++b)
#pragma unroll
        for (int h = 0; h < G; ++h) zi[h] += vq_fix(e[b][h], s[h]);
    }
    float z[G];
#pragma unroll
    for (int h = 0; h < G; ++h) z[h] = ldexpf((float)zi[h], -s[h]);
#pragma unroll
    for (int h = 0; h < 4; ++h) ps.lg[h][i] = h < G ? z[h < G ? h : 0] * sm_scale : 0.f;
  }
  __syncthreads();
  partial_softmax_sum(ps, a, row, i0, nvalid, k, pmz, py);
}

// Workgroup 0 of a row merges the chunk partials into y; workgroups 1.. add the final softmax
// weights of their 256 selected tokens to the accumulated scores.
// With `lse` (log of the softmax denominator over ALL resident tokens, per query head) the weights are the
// paper's own, exp(l_i - lse), not renormalised over the selected set (Sec. 3.2, Eq. 5).
__global__ __launch_bounds__(256) void attend_merge(Layout L, const int32_t* __restrict__ idx,
                                                    const int32_t* __restrict__ count, int32_t k, AttendWs a,
                                                    int nsplit, float* __restrict__ y, float* __restrict__ acc,
                                                    const float* __restrict__ lse, HostShare hs) {
  __shared__ float fm[4], fz[4];
  __shared__ float wgt[4][64];  // nsplit <= 64
  __shared__ float pm[64][4], pz[64][4];
  const int row = blockIdx.y;
  const int cnt = count[row];
  const float* pmz = a.pmz + ((int64_t)row * nsplit * 4) * 2;
  // all chunk (max, sum) pairs are fetched by separate threads in one go, then reduced from LDS
  if (threadIdx.x < 4 * nsplit) {
    const float2 v = reinterpret_cast<const float2*>(pmz)[threadIdx.x];   // index = split*4 + head
    pm[threadIdx.x >> 2][threadIdx.x & 3] = v.x;
    pz[threadIdx.x >> 2][threadIdx.x & 3] = v.y;
  }
  __syncthreads();
  if (threadIdx.x < 4) {
    const int h = threadIdx.x;
    float m = -INFINITY;
    for (int sp = 0; sp < nsplit; ++sp) m = fmaxf(m, pm[sp][h]);
    float z = 0.f;
    for (int sp = 0; sp < nsplit; ++sp) {
      const float ms = pm[sp][h];
      const float e = (ms == -INFINITY) ? 0.f : expf(ms - m);
      wgt[h][sp] = e;
      z += e * pz[sp][h];
    }
    // global normalisation: sum_i exp(l_i - m) v_i / exp(lse - m)
    if (lse != nullptr && h < L.gqa) z = expf(lse[(int64_t)row * L.gqa + h] - m);
    fm[h] = m; fz[h] = z;
  }
  __syncthreads();
  if (blockIdx.x == 0) {
    if (hs.chunks > 0) {
      // the host's partial sums of this row: wait, a bounded number of polls, until the host has stored this
      // step's sequence number (it never stores an older one afterwards)
      if (threadIdx.x == 0) {
        int polls = 0;
        while ((int32_t)(__hip_atomic_load(hs.host_seq + row, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) - hs.seq) < 0) {
          if (++polls >= hs.spin_limit) {
            __hip_atomic_store(hs.err, hs.seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            break;
          }
          __builtin_amdgcn_s_sleep(20);
        }
      }
      __syncthreads();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "");       // nothing read below may come from before the flag
    }
    for (int c = threadIdx.x; c < L.gqa * kHeadDim; c += 256) {
      const int h = c >> 7, d = c & 127;
      float s = 0.f;
      // chunks of the host share: device-side partial (entries the host cannot reach) + the host's partial
      for (int sp = 0; sp < hs.chunks && sp < nsplit; ++sp) {
        const float e = wgt[h][sp];
        if (e != 0.f) {
          const float v = a.py[((int64_t)row * nsplit * 4 + sp * 4 + h) * kHeadDim + d] +
                          __builtin_nontemporal_load(&hs.py[(((int64_t)row * hs.chunks + sp) * 4 + h) * kHeadDim + d]);
          s = fmaf(e, v, s);
        }
      }
      const float* src = a.py + ((int64_t)row * nsplit * 4 + h) * kHeadDim + d;
      for (int s0 = hs.chunks; s0 < nsplit; s0 += 16) {      // 16 independent loads per batch
        float v[16];
#pragma unroll
        for (int x = 0; x < 16; ++x) v[x] = (s0 + x < nsplit) ? src[(int64_t)(s0 + x) * 4 * kHeadDim] : 0.f;
#pragma unroll
        for (int x = 0; x < 16; ++x)
          if (s0 + x < nsplit) s = fmaf(wgt[h][s0 + x], v[x], s);
      }
      y[((int64_t)row * L.gqa + h) * kHeadDim + d] = cnt > 0 ? s / fz[h] : 0.f;
    }
  } else if (acc != nullptr) {
    const int i = (blockIdx.x - 1) * 256 + threadIdx.x;
    if (i < cnt) {
      float wsum = 0.f;
      for (int h = 0; h < L.gqa; ++h) {
        const float p = expf(a.logit[((int64_t)row * 4 + h) * k + i] - fm[h]) / fz[h];
        wsum += fmaxf(p, 1e-30f);
      }
      acc[(int64_t)row * L.cap + idx[(int64_t)row * k + i]] += wsum;
    }
  }
}

// Small per-thread ring of events for the stream fork / join around the gather.
static hipEvent_t next_event(hipError_t* err) {
  thread_local hipEvent_t ring[32];
  thread_local bool made[32] = {false};
  thread_local int cur = 0;
  const int i = cur;
  cur = (cur + 1) & 31;
  *err = hipSuccess;
  if (!made[i]) {
    *err = hipEventCreateWithFlags(&ring[i], hipEventDisableTiming);
    if (*err != hipSuccess) return nullptr;
    made[i] = true;
  }
  return ring[i];
}

int32_t launch_gather(const Layout& L, const int32_t* idx, const int32_t* count, int32_t k, const int32_t* pos,
                      const void* v_host, int64_t host_stride, int64_t n_host_rows, const void* v_hbm,
                      int64_t hbm_stride, void* ws, hipStream_t st, uint64_t* stamps, int first_entry,
                      const Tuning* tune, const HostShare* hs) {
  AttendWs a;
  carve(&a, ws, L, k);
  uint32_t* gpu_seq = hs != nullptr ? hs->gpu_seq : nullptr;
  const uint32_t seq = hs != nullptr ? hs->seq : 0u;
  const Tuning& tn = tune != nullptr ? *tune : tuning();
  int64_t wgs = ((int64_t)k + 15) / 16;                  // one workgroup per 16 rows at most
  // per (sequence, KV head).  About 64 workgroups in total keep enough reads in flight to fill the host
  // link; more only take queue entries in the memory system away from the HBM-bound kernels beside it.
  int64_t lim = tn.gather_wgs > 0 ? tn.gather_wgs : (L.rows >= 64 ? 1 : 64 / L.rows);
  if (wgs > lim) wgs = lim;
  if (wgs * L.rows > kGatherStampPairs) stamps = nullptr;      // more workgroups than the stamp buffer holds
  dim3 g((unsigned)wgs, (unsigned)L.rows);
  const uint4 *vh = (const uint4*)v_host, *vd = (const uint4*)v_hbm;
#define HCA_GATHER(U)                                                                                              \
  gather_values<U><<<g, 256, 0, st>>>(idx, count, k, pos, L.cap, vh, host_stride, n_host_rows, vd, hbm_stride, \
                                      (uint4*)a.vstage, (int)wgs, stamps, first_entry, gpu_seq, seq)
  if (tn.gather_unroll >= 4) HCA_GATHER(4);
  else if (tn.gather_unroll >= 2) HCA_GATHER(2);
  else HCA_GATHER(1);
#undef HCA_GATHER
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

int32_t launch_attend_gathered(const Layout& L, const void* kcache, const void* q, const int32_t* idx,
                               const int32_t* count, int32_t k, float sm_scale, float* y, float* acc_opt,
                               void* ws, hipStream_t st, const float* lse, const HostShare* hs) {
  AttendWs a;
  carve(&a, ws, L, k);
  const int ns = nsplit_of(k);
  if (ns > 64) return HCA_ERR_CAPACITY;
  HostShare h0;
  if (hs != nullptr) h0 = *hs;
  if (h0.chunks > ns) h0.chunks = ns;
  if (ns - h0.chunks > 0) {            // the chunks whose value rows the gather has staged
    dim3 gp((unsigned)(ns - h0.chunks), (unsigned)L.rows);
    if (L.bits == 4)
      attend_partial<4><<<gp, 256, 0, st>>>(L, (const uint8_t*)kcache, (const uint16_t*)q, idx, count, k, sm_scale, a, ns,
                                            h0.chunks);
    else
      attend_partial<2><<<gp, 256, 0, st>>>(L, (const uint8_t*)kcache, (const uint16_t*)q, idx, count, k, sm_scale, a, ns,
                                            h0.chunks);
  }
  dim3 gm((unsigned)(1 + (acc_opt ? ns : 0)), (unsigned)L.rows);
  attend_merge<<<gm, 256, 0, st>>>(L, idx, count, k, a, ns, y, acc_opt, lse, h0);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

int host_share_chunks(int32_t k, int want) {
  const int ns = nsplit_of(k);
  return want < 0 ? 0 : (want > ns ? ns : want);
}
size_t host_share_p_bytes(const Layout& L, int chunks) { return (size_t)L.rows * chunks * 4 * kChunk * sizeof(float); }
size_t host_share_vrow_bytes(const Layout& L, int chunks) { return (size_t)L.rows * chunks * kChunk * sizeof(int32_t); }
size_t host_share_py_bytes(const Layout& L, int chunks) { return (size_t)L.rows * chunks * 4 * kHeadDim * sizeof(float); }

int32_t launch_attend_host_chunks(const Layout& L, const void* kcache, const void* q, const int32_t* idx,
                                  const int32_t* count, int32_t k, const int32_t* pos, int64_t n_host_rows,
                                  const void* v_hbm, int64_t hbm_stride, float sm_scale, void* ws, const HostShare& hs,
                                  hipStream_t st) {
  AttendWs a;
  carve(&a, ws, L, k);
  const int ns = nsplit_of(k);
  if (ns > 64 || hs.chunks < 1 || hs.chunks > ns) return HCA_ERR_CAPACITY;
  dim3 gp((unsigned)hs.chunks, (unsigned)L.rows);
  if (L.bits == 4)
    attend_host_chunks<4><<<gp, 256, 0, st>>>(L, (const uint8_t*)kcache, (const uint16_t*)q, idx, count, k, pos,
                                              n_host_rows, (const uint16_t*)v_hbm, hbm_stride, sm_scale, a, ns, hs);
  else
    attend_host_chunks<2><<<gp, 256, 0, st>>>(L, (const uint8_t*)kcache, (const uint16_t*)q, idx, count, k, pos,
                                              n_host_rows, (const uint16_t*)v_hbm, hbm_stride, sm_scale, a, ns, hs);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

int32_t launch_vq_attend_gathered(const Layout& L, int g, int c, const uint8_t* pcache, const float* lut,
                                  const int32_t* idx, const int32_t* count, int32_t k, float sm_scale, float* y,
                                  float* acc_opt, void* ws, hipStream_t st) {
  AttendWs a;
  carve(&a, ws, L, k);
  const int ns = nsplit_of(k);
  if (ns > 64) return HCA_ERR_CAPACITY;
  dim3 gp((unsigned)ns, (unsigned)L.rows);
#define HCA_VQ_PARTIAL(GQ)                                                                                               \
  do {                                                                                                                   \
    if (vq_is_wide(L, g, c)) vq_attend_partial<GQ, true><<<gp, 256, 0, st>>>(g, c, L.cap, pcache, lut, idx, count, k, sm_scale, a, ns); \
    else vq_attend_partial<GQ, false><<<gp, 256, 0, st>>>(g, c, L.cap, pcache, lut, idx, count, k, sm_scale, a, ns);               \
  } while (0)
  if (L.gqa == 4) HCA_VQ_PARTIAL(4);
  else if (L.gqa == 2) HCA_VQ_PARTIAL(2);
  else HCA_VQ_PARTIAL(1);
#undef HCA_VQ_PARTIAL
  dim3 gm((unsigned)(1 + (acc_opt ? ns : 0)), (unsigned)L.rows);
  attend_merge<<<gm, 256, 0, st>>>(L, idx, count, k, a, ns, y, acc_opt, nullptr, HostShare{});
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

// The paper's split (Sec. 3.2 "CPU part", Sec. 3.3 "Communication overhead"): only the selected tokens'
// value-row numbers and weights leave the GPU (2 bytes per weight), the host forms the weighted sum.
// One workgroup per chunk of 256 selected tokens merges the chunk (max, sum) pairs of the row and writes
// fp16 weights [row * G + h][k], value rows [row][k] and, optionally, the accumulated scores.
__global__ __launch_bounds__(256) void weights_finalize(Layout L, const int32_t* __restrict__ idx,
                                                        const int32_t* __restrict__ count, int32_t k,
                                                        const int32_t* __restrict__ pos, AttendWs a, int nsplit,
                                                        const float* __restrict__ lse, uint16_t* __restrict__ w_out,
                                                        int32_t* __restrict__ vrow_out, float* __restrict__ acc) {
  __shared__ float fm[4], fz[4];
  __shared__ float pm[64][4], pz[64][4];
  const int row = blockIdx.y;
  const int cnt = count[row];
  const float* pmz = a.pmz + ((int64_t)row * nsplit * 4) * 2;
  if (threadIdx.x < 4 * nsplit) {
    const float2 v = reinterpret_cast<const float2*>(pmz)[threadIdx.x];
    pm[threadIdx.x >> 2][threadIdx.x & 3] = v.x;
    pz[threadIdx.x >> 2][threadIdx.x & 3] = v.y;
  }
  __syncthreads();
  if (threadIdx.x < 4) {
    const int h = threadIdx.x;
    float m = -INFINITY;
    for (int sp = 0; sp < nsplit; ++sp) m = fmaxf(m, pm[sp][h]);
    float z = 0.f;
    for (int sp = 0; sp < nsplit; ++sp) {
      const float ms = pm[sp][h];
      z += (ms == -INFINITY) ? 0.f : expf(ms - m) * pz[sp][h];
    }
    if (lse != nullptr && h < L.gqa) z = expf(lse[(int64_t)row * L.gqa + h] - m);
    fm[h] = m; fz[h] = z;
  }
  __syncthreads();
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= k) return;
  const bool live = i < cnt;
  float wsum = 0.f;
  for (int h = 0; h < L.gqa; ++h) {
    const float p = live ? expf(a.logit[((int64_t)row * 4 + h) * k + i] - fm[h]) / fz[h] : 0.f;
    w_out[((int64_t)row * L.gqa + h) * k + i] = f2h_bits(p);
    wsum += fmaxf(p, 1e-30f);
  }
  const int32_t slot = live ? idx[(int64_t)row * k + i] : 0;
  vrow_out[(int64_t)row * k + i] = live ? pos[(int64_t)row * L.cap + slot] : -1;
  if (live && acc != nullptr) acc[(int64_t)row * L.cap + slot] += wsum;
}

int32_t launch_attend_weights(const Layout& L, const void* kcache, const void* q, const int32_t* idx,
                              const int32_t* count, int32_t k, const int32_t* pos, float sm_scale, const float* lse,
                              void* w_out, int32_t* vrow_out, float* acc_opt, void* ws, hipStream_t st) {
  AttendWs a;
  carve(&a, ws, L, k);
  const int ns = nsplit_of(k);
  if (ns > 64) return HCA_ERR_CAPACITY;
  dim3 gp((unsigned)ns, (unsigned)L.rows);
  if (L.bits == 4)
    attend_partial<4, false><<<gp, 256, 0, st>>>(L, (const uint8_t*)kcache, (const uint16_t*)q, idx, count, k, sm_scale, a, ns, 0);
  else
    attend_partial<2, false><<<gp, 256, 0, st>>>(L, (const uint8_t*)kcache, (const uint16_t*)q, idx, count, k, sm_scale, a, ns, 0);
  weights_finalize<<<gp, 256, 0, st>>>(L, idx, count, k, pos, a, ns, lse, (uint16_t*)w_out, vrow_out, acc_opt);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

int32_t launch_attend(const Layout& L, const void* kcache, const void* q, const int32_t* idx,
                      const int32_t* count, int32_t k, const int32_t* pos, const void* v_host,
                      int64_t host_stride, int64_t n_host_rows, const void* v_hbm, int64_t hbm_stride,
                      float sm_scale, float* y, float* acc_opt, void* ws, hipStream_t gst, hipStream_t st) {
  if (nsplit_of(k) > 64) return HCA_ERR_CAPACITY;
  if (gst != st) {
    hipError_t e;
    hipEvent_t ev = next_event(&e);
    if (e != hipSuccess) return hip_fail(e);
    HCA_HIP(hipEventRecord(ev, st));
    HCA_HIP(hipStreamWaitEvent(gst, ev, 0));
  }
  int32_t rc = launch_gather(L, idx, count, k, pos, v_host, host_stride, n_host_rows, v_hbm, hbm_stride, ws, gst);
  if (rc != HCA_OK) return rc;
  if (gst != st) {
    hipError_t e;
    hipEvent_t ev = next_event(&e);
    if (e != hipSuccess) return hip_fail(e);
    HCA_HIP(hipEventRecord(ev, gst));
    HCA_HIP(hipStreamWaitEvent(st, ev, 0));
  }
  return launch_attend_gathered(L, kcache, q, idx, count, k, sm_scale, y, acc_opt, ws, st);
}

}  // namespace hca
