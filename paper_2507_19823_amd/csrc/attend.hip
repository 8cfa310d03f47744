// Step 3b: gather of the selected value rows (pinned host memory and / or an HBM slice) and the
// softmax-weighted sum over the selected set (Eq. 5), plus the accumulated-score update.
#include "hca_internal.h"

namespace hca {

constexpr int kChunk = 256;  // selected tokens per workgroup of the partial kernel

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
// pinned host memory over the host link (zero-copy), the others from the HBM slice.
__global__ __launch_bounds__(256) void gather_values(const int32_t* __restrict__ idx, const int32_t* __restrict__ count,
                                                     int32_t k, const int32_t* __restrict__ pos, int64_t cap,
                                                     const uint4* __restrict__ v_host, int64_t host_stride,
                                                     int64_t n_host_rows, const uint4* __restrict__ v_hbm,
                                                     int64_t hbm_stride, uint4* __restrict__ vstage) {
  const int row = blockIdx.y;
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t i = gid >> 4;
  const int part = (int)(gid & 15);
  if (i >= count[row]) return;
  const int32_t slot = idx[(int64_t)row * k + i];
  const int64_t v = pos[(int64_t)row * cap + slot];
  const uint4* src = (v < n_host_rows) ? v_host + ((int64_t)row * host_stride + v) * 16
                                       : v_hbm + ((int64_t)row * hbm_stride + (v - n_host_rows)) * 16;
  vstage[((int64_t)row * k + i) * 16 + part] = src[part];
}

template <int BITS>
__global__ __launch_bounds__(256) void attend_partial(Layout L, const uint8_t* __restrict__ kcache,
                                                      const uint16_t* __restrict__ q, const int32_t* __restrict__ idx,
                                                      const int32_t* __restrict__ count, int32_t k, float sm_scale,
                                                      AttendWs a, int nsplit) {
  __shared__ QShared sh;
  __shared__ float lg[4][kChunk];
  __shared__ float red[4][4][kHeadDim];
  __shared__ float hm[4], hz[4];
  const int row = blockIdx.y, split = blockIdx.x;
  const int cnt = count[row];
  const int i0 = split * kChunk;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int t = lane & 15, j = lane >> 4;
  float* pmz = a.pmz + (((int64_t)row * nsplit + split) * 4) * 2;
  float* py = a.py + (((int64_t)row * nsplit + split) * 4) * kHeadDim;
  if (i0 >= cnt) {  // empty chunk: neutral partial
    if (threadIdx.x < 4) { pmz[2 * threadIdx.x] = -INFINITY; pmz[2 * threadIdx.x + 1] = 0.f; }
    for (int c = threadIdx.x; c < 4 * kHeadDim; c += 256) py[c] = 0.f;
    return;
  }
  const int nvalid = (cnt - i0 < kChunk) ? cnt - i0 : kChunk;
  load_query(q, row, L.gqa, L.group, &sh);
  QOperand<BITS> op;
  build_operand<BITS>(&sh, &op);
  const uint8_t* crow = kcache + (int64_t)row * L.codes_row_bytes();
  const uint8_t* mrow = kcache + L.meta_off + (int64_t)row * L.meta_row_bytes();
  const int32_t* ridx = idx + (int64_t)row * k;

  // 1. logits of the chunk: wave w scores tiles w, w+4, ... (16 selected tokens each)
  for (int tile = w; tile * 16 < nvalid; tile += 4) {
    const int i = tile * 16 + t;
    const int ii = i < nvalid ? i : nvalid - 1;
    const int64_t slot = ridx[i0 + ii];
    float zv;
    if constexpr (BITS == 4) {
      const int64_t blk = slot >> 4;
      const int tl = (int)(slot & 15);
      const uint4 wv = *reinterpret_cast<const uint4*>(crow + blk * kBlockBytes + (tl + 16 * j) * 16);
      const uint4 mv = *reinterpret_cast<const uint4*>(mrow + blk * kMetaBytes + tl * 16);
      zv = score_block4(op, wv, mv);
    } else {
      const int64_t blk = slot >> 5;
      const int u = (int)((slot >> 4) & 1), tl = (int)(slot & 15);
      const uint2 wv = *reinterpret_cast<const uint2*>(crow + blk * kBlockBytes + (tl + 16 * j) * 16 + 8 * u);
      const uint2 mv = *reinterpret_cast<const uint2*>(mrow + blk * kMetaBytes + (16 * u + tl) * 8);
      zv = score_tile2(op, wv.x, wv.y, mv);
    }
    // lane (t, hd = j) holds z~ of head j for selected token i
    lg[j][i] = zv * sm_scale;
  }
  __syncthreads();

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

  // 3. weighted value sum: wave w takes tokens w, w+4, ...; lane owns channels 2*lane, 2*lane+1
  float acc[4][2] = {{0.f, 0.f}, {0.f, 0.f}, {0.f, 0.f}, {0.f, 0.f}};
  const uint32_t* vs = reinterpret_cast<const uint32_t*>(a.vstage) + ((int64_t)row * k + i0) * 64 + lane;
  for (int i = w; i < nvalid; i += 4) {
    const uint32_t pr = vs[(int64_t)i * 64];
    const float v0 = h2f(pr & 0xffffu), v1 = h2f(pr >> 16);
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      const float p = lg[h][i];
      acc[h][0] = fmaf(p, v0, acc[h][0]);
      acc[h][1] = fmaf(p, v1, acc[h][1]);
    }
  }
#pragma unroll
  for (int h = 0; h < 4; ++h) { red[w][h][2 * lane] = acc[h][0]; red[w][h][2 * lane + 1] = acc[h][1]; }
  __syncthreads();
  for (int c = threadIdx.x; c < 4 * kHeadDim; c += 256) {
    const int h = c >> 7, d = c & 127;
    py[c] = (red[0][h][d] + red[1][h][d]) + (red[2][h][d] + red[3][h][d]);
  }
  if (threadIdx.x < 4) { pmz[2 * threadIdx.x] = hm[threadIdx.x]; pmz[2 * threadIdx.x + 1] = hz[threadIdx.x]; }
}

// Workgroup 0 of a row merges the chunk partials into y; workgroups 1.. add the final softmax
// weights of their 256 selected tokens to the accumulated scores.
__global__ __launch_bounds__(256) void attend_merge(Layout L, const int32_t* __restrict__ idx,
                                                    const int32_t* __restrict__ count, int32_t k, AttendWs a,
                                                    int nsplit, float* __restrict__ y, float* __restrict__ acc) {
  __shared__ float fm[4], fz[4];
  __shared__ float wgt[4][64];  // nsplit <= 64
  const int row = blockIdx.y;
  const int cnt = count[row];
  const float* pmz = a.pmz + ((int64_t)row * nsplit * 4) * 2;
  if (threadIdx.x < 4) {
    const int h = threadIdx.x;
    float m = -INFINITY;
    for (int s = 0; s < nsplit; ++s) m = fmaxf(m, pmz[(s * 4 + h) * 2]);
    float z = 0.f;
    for (int s = 0; s < nsplit; ++s) {
      const float ms = pmz[(s * 4 + h) * 2];
      const float e = (ms == -INFINITY) ? 0.f : expf(ms - m);
      wgt[h][s] = e;
      z += e * pmz[(s * 4 + h) * 2 + 1];
    }
    fm[h] = m; fz[h] = z;
  }
  __syncthreads();
  if (blockIdx.x == 0) {
    for (int c = threadIdx.x; c < L.gqa * kHeadDim; c += 256) {
      const int h = c >> 7, d = c & 127;
      float s = 0.f;
      for (int sp = 0; sp < nsplit; ++sp)
        s = fmaf(wgt[h][sp], a.py[(((int64_t)row * nsplit + sp) * 4 + h) * kHeadDim + d], s);
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

int32_t launch_attend(const Layout& L, const void* kcache, const void* q, const int32_t* idx,
                      const int32_t* count, int32_t k, const int32_t* pos, const void* v_host,
                      int64_t host_stride, int64_t n_host_rows, const void* v_hbm, int64_t hbm_stride,
                      float sm_scale, float* y, float* acc_opt, void* ws, hipStream_t gst, hipStream_t st) {
  AttendWs a;
  carve(&a, ws, L, k);
  const int ns = nsplit_of(k);
  if (ns > 64) return HCA_ERR_CAPACITY;
  if (gst != st) {
    hipError_t e;
    hipEvent_t ev = next_event(&e);
    if (e != hipSuccess) return hip_fail(e);
    HCA_HIP(hipEventRecord(ev, st));
    HCA_HIP(hipStreamWaitEvent(gst, ev, 0));
  }
  {
    dim3 g((unsigned)(((int64_t)k * 16 + 255) / 256), (unsigned)L.rows);
    gather_values<<<g, 256, 0, gst>>>(idx, count, k, pos, L.cap, (const uint4*)v_host, host_stride, n_host_rows,
                                      (const uint4*)v_hbm, hbm_stride, (uint4*)a.vstage);
    HCA_HIP(hipGetLastError());
  }
  if (gst != st) {
    hipError_t e;
    hipEvent_t ev = next_event(&e);
    if (e != hipSuccess) return hip_fail(e);
    HCA_HIP(hipEventRecord(ev, gst));
    HCA_HIP(hipStreamWaitEvent(st, ev, 0));
  }
  dim3 gp((unsigned)ns, (unsigned)L.rows);
  if (L.bits == 4)
    attend_partial<4><<<gp, 256, 0, st>>>(L, (const uint8_t*)kcache, (const uint16_t*)q, idx, count, k, sm_scale, a, ns);
  else
    attend_partial<2><<<gp, 256, 0, st>>>(L, (const uint8_t*)kcache, (const uint16_t*)q, idx, count, k, sm_scale, a, ns);
  dim3 gm((unsigned)(1 + (acc_opt ? ns : 0)), (unsigned)L.rows);
  attend_merge<<<gm, 256, 0, st>>>(L, idx, count, k, a, ns, y, acc_opt);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

}  // namespace hca
