// Exact selection engine and step 3a (top-k).  Per row, a 3-pass radix select (11 + 11 + 10
// bits of an order-preserving key) finds the threshold key T and how many slots equal to T
// are needed; a counting pass plus a chunk prefix then lets an ordered pass emit the
// selected slots in ascending order with ties resolved towards the lower slot:
//   selected(j) = key_j > T  or  (key_j == T and #{i < j : key_i == T} < r_eq)
//   position(j) = #{i < j : key_i > T} + min(#{i < j : key_i == T}, r_eq)
// This is the sorted prefix Pi_k of Sec. 3.2 without sorting.
#include "hca_internal.h"

namespace hca {

constexpr int kBins = 2048;

__device__ __forceinline__ int pass_shift(int p) { return p == 0 ? 21 : (p == 1 ? 10 : 0); }

size_t select_workspace_bytes(int rows, int64_t nmax) {
  (void)nmax;
  size_t b = 0;
  b += align_up((int64_t)rows * 3 * kBins * 4, 256);
  b += align_up((int64_t)rows * 4 * 4, 256);
  b += 2 * align_up((int64_t)rows * 1024 * 2 * 4, 256);
  return b;
}

void select_plan(SelectPlan* p, void* ws, int rows, int64_t nmax) {
  int64_t chunk = align_up((nmax + 1023) / 1024, 1024);
  if (chunk < 4096) chunk = 4096;
  p->chunk = chunk;
  p->nchunks = (int32_t)((nmax + chunk - 1) / chunk);
  if (p->nchunks < 1) p->nchunks = 1;
  uint8_t* w = (uint8_t*)ws;
  p->hist = (uint32_t*)w;   w += align_up((int64_t)rows * 3 * kBins * 4, 256);
  p->state = (uint32_t*)w;  w += align_up((int64_t)rows * 4 * 4, 256);
  p->ccount = (uint32_t*)w; w += align_up((int64_t)rows * 1024 * 2 * 4, 256);
  p->coff = (uint32_t*)w;
}

__global__ void sel_init(uint32_t* hist, uint32_t* state, int rows, int n_kv_heads, SelRows sr) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < (int64_t)rows * 3 * kBins) hist[i] = 0;
  if (i < rows) {
    const int64_t want = sr.want[i / n_kv_heads];
    state[4 * i + 0] = (want == 0) ? 0xffffffffu : 0u;
    state[4 * i + 1] = want > 0 ? (uint32_t)want : 0u;
  }
}

template <int PASS>
__global__ __launch_bounds__(256) void sel_hist(const float* __restrict__ vals, int64_t stride, int64_t chunk,
                                                int n_kv_heads, SelRows sr, uint32_t* __restrict__ hist,
                                                const uint32_t* __restrict__ state) {
  __shared__ uint32_t lh[kBins];
  const int row = blockIdx.y;
  const int64_t nsel = sr.nsel[row / n_kv_heads];
  if (sr.want[row / n_kv_heads] <= 0) return;
  const int64_t c0 = (int64_t)blockIdx.x * chunk;
  if (c0 >= nsel) return;
  int64_t c1 = c0 + chunk;
  if (c1 > nsel) c1 = nsel;
  for (int i = threadIdx.x; i < kBins; i += 256) lh[i] = 0;
  __syncthreads();
  const uint32_t prefix = state[4 * row];
  const float* v = vals + (int64_t)row * stride;
  for (int64_t j = c0 + threadIdx.x; j < c1; j += 256) {
    const uint32_t key = order_key(v[j]);
    if (PASS == 0) {
      atomicAdd(&lh[key >> 21], 1u);
    } else if (PASS == 1) {
      if ((key >> 21) == (prefix >> 21)) atomicAdd(&lh[(key >> 10) & 2047u], 1u);
    } else {
      if ((key >> 10) == (prefix >> 10)) atomicAdd(&lh[key & 1023u], 1u);
    }
  }
  __syncthreads();
  uint32_t* gh = hist + ((int64_t)row * 3 + PASS) * kBins;
  for (int i = threadIdx.x; i < kBins; i += 256) {
    const uint32_t c = lh[i];
    if (c) atomicAdd(&gh[i], c);
  }
}

// One workgroup per row: picks the bin holding the `remaining`-th largest key.
template <int PASS>
__global__ __launch_bounds__(256) void sel_scan(const uint32_t* __restrict__ hist, uint32_t* __restrict__ state,
                                                int n_kv_heads, SelRows sr) {
  __shared__ uint32_t s[256];
  const int row = blockIdx.x;
  if (sr.want[row / n_kv_heads] <= 0) return;
  const uint32_t remaining = state[4 * row + 1];
  const uint32_t* gh = hist + ((int64_t)row * 3 + PASS) * kBins;
  const int t = threadIdx.x;
  uint32_t h[8];
  uint32_t sum = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) { h[i] = gh[8 * t + i]; sum += h[i]; }
  s[t] = sum;
  __syncthreads();
  // inclusive suffix scan over threads (Hillis-Steele)
  for (int o = 1; o < 256; o <<= 1) {
    const uint32_t add = (t + o < 256) ? s[t + o] : 0;
    __syncthreads();
    s[t] += add;
    __syncthreads();
  }
  uint32_t running = s[t] - sum;  // keys in bins above this thread's range
#pragma unroll
  for (int i = 7; i >= 0; --i) {
    if (running < remaining && remaining <= running + h[i]) {
      state[4 * row + 0] |= (uint32_t)(8 * t + i) << pass_shift(PASS);
      state[4 * row + 1] = remaining - running;
    }
    running += h[i];
  }
}

__global__ __launch_bounds__(256) void sel_count(const float* __restrict__ vals, int64_t stride, int64_t chunk,
                                                 int n_kv_heads, SelRows sr, const uint32_t* __restrict__ state,
                                                 uint32_t* __restrict__ ccount) {
  __shared__ uint32_t red[2][4];
  const int row = blockIdx.y;
  if (sr.want[row / n_kv_heads] < 0) return;
  const int64_t nsel = sr.nsel[row / n_kv_heads];
  const int64_t c0 = (int64_t)blockIdx.x * chunk;
  int64_t c1 = c0 + chunk;
  if (c1 > nsel) c1 = nsel;
  const uint32_t T = state[4 * row];
  const float* v = vals + (int64_t)row * stride;
  uint32_t gt = 0, eq = 0;
  for (int64_t j = c0 + threadIdx.x; j < c1; j += 256) {
    const uint32_t key = order_key(v[j]);
    gt += key > T;
    eq += key == T;
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) { gt += __shfl_xor(gt, o); eq += __shfl_xor(eq, o); }
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { red[0][w] = gt; red[1][w] = eq; }
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t* o = ccount + ((int64_t)row * gridDim.x + blockIdx.x) * 2;
    o[0] = red[0][0] + red[0][1] + red[0][2] + red[0][3];
    o[1] = red[1][0] + red[1][1] + red[1][2] + red[1][3];
  }
}

// Exclusive prefix over the chunks of a row (nchunks <= 1024).
__global__ __launch_bounds__(256) void sel_offsets(const uint32_t* __restrict__ ccount, uint32_t* __restrict__ coff,
                                                   int nchunks, int n_kv_heads, SelRows sr) {
  __shared__ uint32_t s[2][256];
  const int row = blockIdx.x;
  if (sr.want[row / n_kv_heads] < 0) return;
  const int t = threadIdx.x;
  uint32_t g[4], e[4], sg = 0, se = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = 4 * t + i;
    g[i] = c < nchunks ? ccount[((int64_t)row * nchunks + c) * 2] : 0;
    e[i] = c < nchunks ? ccount[((int64_t)row * nchunks + c) * 2 + 1] : 0;
    sg += g[i]; se += e[i];
  }
  s[0][t] = sg; s[1][t] = se;
  __syncthreads();
  for (int o = 1; o < 256; o <<= 1) {
    const uint32_t ag = t >= o ? s[0][t - o] : 0, ae = t >= o ? s[1][t - o] : 0;
    __syncthreads();
    s[0][t] += ag; s[1][t] += ae;
    __syncthreads();
  }
  uint32_t rg = s[0][t] - sg, re = s[1][t] - se;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = 4 * t + i;
    if (c < nchunks) {
      coff[((int64_t)row * nchunks + c) * 2] = rg;
      coff[((int64_t)row * nchunks + c) * 2 + 1] = re;
    }
    rg += g[i]; re += e[i];
  }
}

int32_t select_run(const SelectPlan& p, const float* vals, int64_t stride, int rows, int n_kv_heads,
                   const SelRows& sr, hipStream_t st) {
  {
    const int64_t n = (int64_t)rows * 3 * kBins;
    sel_init<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(p.hist, p.state, rows, n_kv_heads, sr);
  }
  dim3 g((unsigned)p.nchunks, (unsigned)rows);
  sel_hist<0><<<g, 256, 0, st>>>(vals, stride, p.chunk, n_kv_heads, sr, p.hist, p.state);
  sel_scan<0><<<rows, 256, 0, st>>>(p.hist, p.state, n_kv_heads, sr);
  sel_hist<1><<<g, 256, 0, st>>>(vals, stride, p.chunk, n_kv_heads, sr, p.hist, p.state);
  sel_scan<1><<<rows, 256, 0, st>>>(p.hist, p.state, n_kv_heads, sr);
  sel_hist<2><<<g, 256, 0, st>>>(vals, stride, p.chunk, n_kv_heads, sr, p.hist, p.state);
  sel_scan<2><<<rows, 256, 0, st>>>(p.hist, p.state, n_kv_heads, sr);
  sel_count<<<g, 256, 0, st>>>(vals, stride, p.chunk, n_kv_heads, sr, p.state, p.ccount);
  sel_offsets<<<rows, 256, 0, st>>>(p.ccount, p.coff, p.nchunks, n_kv_heads, sr);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

// Ordered emit for top-k: each workgroup walks its chunk in slot order, 1024 slots per step
// (4 consecutive slots per thread), and writes the selected slots at their final positions.
__global__ __launch_bounds__(256) void topk_emit(const float* __restrict__ vals, int64_t stride, int64_t chunk,
                                                 int nchunks, int n_kv_heads, SelRows sr,
                                                 const uint32_t* __restrict__ state, const uint32_t* __restrict__ coff,
                                                 int32_t k, int32_t* __restrict__ idx, int32_t* __restrict__ count) {
  __shared__ uint32_t wsum[2][4];
  const int row = blockIdx.y;
  const int64_t want = sr.want[row / n_kv_heads];
  if (blockIdx.x == 0 && threadIdx.x == 0) count[row] = want > 0 ? (int32_t)want : 0;
  if (want <= 0) return;
  const int64_t nsel = sr.nsel[row / n_kv_heads];
  const int64_t c0 = (int64_t)blockIdx.x * chunk;
  if (c0 >= nsel) return;
  int64_t c1 = c0 + chunk;
  if (c1 > nsel) c1 = nsel;
  const uint32_t T = state[4 * row], req = state[4 * row + 1];
  uint32_t base_g = coff[((int64_t)row * nchunks + blockIdx.x) * 2];
  uint32_t base_e = coff[((int64_t)row * nchunks + blockIdx.x) * 2 + 1];
  const float* v = vals + (int64_t)row * stride;
  int32_t* out = idx + (int64_t)row * k;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  for (int64_t s0 = c0; s0 < c1; s0 += 1024) {
    const int64_t j0 = s0 + 4 * threadIdx.x;
    bool fg[4], fe[4];
    uint32_t ng = 0, ne = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t j = j0 + i;
      uint32_t key = 0;
      const bool in = j < c1;
      if (in) key = order_key(v[j]);
      fg[i] = in && key > T;
      fe[i] = in && key == T;
      ng += fg[i]; ne += fe[i];
    }
    // exclusive scan of (ng, ne) across the workgroup
    uint32_t ig = ng, ie = ne;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t ag = __shfl_up(ig, o), ae = __shfl_up(ie, o);
      if (lane >= o) { ig += ag; ie += ae; }
    }
    if (lane == 63) { wsum[0][w] = ig; wsum[1][w] = ie; }
    __syncthreads();
    uint32_t pg = base_g + ig - ng, pe = base_e + ie - ne;
    for (int x = 0; x < w; ++x) { pg += wsum[0][x]; pe += wsum[1][x]; }
    const uint32_t tot_g = wsum[0][0] + wsum[0][1] + wsum[0][2] + wsum[0][3];
    const uint32_t tot_e = wsum[1][0] + wsum[1][1] + wsum[1][2] + wsum[1][3];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (fg[i] || (fe[i] && pe < req)) out[pg + (pe < req ? pe : req)] = (int32_t)(j0 + i);
      pg += fg[i]; pe += fe[i];
    }
    base_g += tot_g; base_e += tot_e;
    __syncthreads();
  }
}

int32_t launch_topk(const Layout& L, const float* sel, const NRes& nr, int64_t nmax, int32_t k,
                    int32_t* idx, int32_t* count, void* ws, hipStream_t st) {
  SelRows sr;
  for (int b = 0; b < kMaxBatch; ++b) { sr.nsel[b] = 0; sr.want[b] = -1; }
  for (int b = 0; b < L.batch; ++b) {
    sr.nsel[b] = nr.n[b];
    sr.want[b] = nr.n[b] < k ? nr.n[b] : k;
    if (sr.want[b] == 0) sr.want[b] = -1;
  }
  SelectPlan p;
  select_plan(&p, ws, L.rows, nmax > 0 ? nmax : 1);
  if (nmax > 0) {
    int32_t rc = select_run(p, sel, L.cap, L.rows, L.n_kv_heads, sr, st);
    if (rc != HCA_OK) return rc;
  }
  dim3 g((unsigned)p.nchunks, (unsigned)L.rows);
  topk_emit<<<g, 256, 0, st>>>(sel, L.cap, p.chunk, p.nchunks, L.n_kv_heads, sr, p.state, p.coff, k, idx, count);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

}  // namespace hca
