// Exact selection engine and step 3a (top-k).  Per row, a 3-pass radix select (11 + 11 + 10
// bits of an order-preserving key) finds the threshold key T and how many slots equal to T
// are needed; a counting pass plus a chunk prefix then lets an ordered pass emit the
// selected slots in ascending order with ties resolved towards the lower slot:
//   selected(j) = key_j > T  or  (key_j == T and #{i < j : key_i == T} < r_eq)
//   position(j) = #{i < j : key_i > T} + min(#{i < j : key_i == T}, r_eq)
// This is the sorted prefix Pi_k of Sec. 3.2 without sorting.  The engine serves the eviction's keep-set, whose
// values are accumulated softmax weights: a first counting pass against 0 settles T for every row whose
// wanted-th largest value is 0 (sel_try_zero), and the radix passes skip those rows.
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
    state[4 * i + 2] = 0xffffffffu;          // lowest slot that is not selected (filled in by the eviction's ordered pass)
    state[4 * i + 3] = 0u;                   // 1: threshold found by the zero-threshold shortcut, the radix passes skip the row
  }
}

template <int PASS>
__global__ __launch_bounds__(256) void sel_hist(const float* __restrict__ vals, int64_t stride, int64_t chunk,
                                                int n_kv_heads, SelRows sr, uint32_t* __restrict__ hist,
                                                const uint32_t* __restrict__ state) {
  __shared__ uint32_t lh[kBins];
  const int row = blockIdx.y;
  const int64_t nsel = sr.nsel[row / n_kv_heads];
  if (sr.want[row / n_kv_heads] <= 0 || state[4 * row + 3] != 0) return;
  const int64_t c0 = (int64_t)blockIdx.x * chunk;
  if (c0 >= nsel) return;
  int64_t c1 = c0 + chunk;
  if (c1 > nsel) c1 = nsel;
  for (int i = threadIdx.x; i < kBins; i += 256) lh[i] = 0;
  __syncthreads();
  const uint32_t prefix = state[4 * row];
  const float* v = vals + (int64_t)row * stride;
  const int lane = threadIdx.x & 63;
  for (int64_t j0 = c0; j0 < c1; j0 += 256) {
    const int64_t j = j0 + threadIdx.x;
    bool hit = j < c1;
    uint32_t bin = 0;
    if (hit) {
      const uint32_t key = order_key(v[j]);
      if (PASS == 0) {
        bin = key >> 21;
      } else if (PASS == 1) {
        hit = (key >> 21) == (prefix >> 21);
        bin = (key >> 10) & 2047u;
      } else {
        hit = (key >> 10) == (prefix >> 10);
        bin = key & 1023u;
      }
    }
    // accumulated scores are mostly equal (0), so a whole wave usually lands in one bin: one
    // atomic for the wave instead of 64 on the same LDS word
    const uint64_t m = __ballot(hit);
    if (m != 0) {
      const int leader = __ffsll((unsigned long long)m) - 1;
      const uint32_t b0 = __shfl(bin, leader);
      if (__ballot(hit && bin != b0) == 0) {
        if (lane == leader) atomicAdd(&lh[b0], (uint32_t)__popcll(m));
      } else if (hit) {
        atomicAdd(&lh[bin], 1u);
      }
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
  if (sr.want[row / n_kv_heads] <= 0 || state[4 * row + 3] != 0) return;
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

// AT_ZERO: the counts are taken against the key of +0.0f, before any radix pass (the shortcut below); otherwise
// against the row's threshold, and rows that the shortcut resolved keep the counts they already have.
template <bool AT_ZERO>
__global__ __launch_bounds__(256) void sel_count(const float* __restrict__ vals, int64_t stride, int64_t chunk,
                                                 int n_kv_heads, SelRows sr, const uint32_t* __restrict__ state,
                                                 uint32_t* __restrict__ ccount) {
  __shared__ uint32_t red[2][4];
  const int row = blockIdx.y;
  if (sr.want[row / n_kv_heads] < 0) return;
  if (!AT_ZERO && state[4 * row + 3] != 0) return;
  const int64_t nsel = sr.nsel[row / n_kv_heads];
  const int64_t c0 = (int64_t)blockIdx.x * chunk;
  int64_t c1 = c0 + chunk;
  if (c1 > nsel) c1 = nsel;
  const uint32_t T = AT_ZERO ? order_key(0.0f) : state[4 * row];
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

// The zero-threshold shortcut.  Accumulated scores are sums of softmax weights: never negative, and exactly 0 for
// every token that was never selected - most of a long context.  When fewer than `want` slots lie above 0 and the
// zeros make up the rest, the want-th largest key is the key of +0.0f and the number of zeros to take is
// want - #(above 0): exactly what the three radix passes would find, from one pass whose per-chunk counts are also
// the ones the ordered pass needs.  One workgroup per row sums the chunk counts and decides.
__global__ __launch_bounds__(256) void sel_try_zero(const uint32_t* __restrict__ ccount, uint32_t* __restrict__ state,
                                                    int nchunks, int n_kv_heads, SelRows sr) {
  __shared__ uint32_t s[2][256];
  const int row = blockIdx.x;
  const int64_t want = sr.want[row / n_kv_heads];
  if (want <= 0) return;
  const int t = threadIdx.x;
  uint32_t g = 0, e = 0;
  for (int c = t; c < nchunks; c += 256) {
    g += ccount[((int64_t)row * nchunks + c) * 2];
    e += ccount[((int64_t)row * nchunks + c) * 2 + 1];
  }
  s[0][t] = g; s[1][t] = e;
  __syncthreads();
  for (int o = 128; o >= 1; o >>= 1) {
    if (t < o) { s[0][t] += s[0][t + o]; s[1][t] += s[1][t + o]; }
    __syncthreads();
  }
  if (t == 0) {
    const uint64_t above = s[0][0], zeros = s[1][0];
    if (above < (uint64_t)want && (uint64_t)want <= above + zeros) {
      state[4 * row + 0] = order_key(0.0f);
      state[4 * row + 1] = (uint32_t)((uint64_t)want - above);
      state[4 * row + 3] = 1u;
    }
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
  sel_count<true><<<g, 256, 0, st>>>(vals, stride, p.chunk, n_kv_heads, sr, p.state, p.ccount);
  sel_try_zero<<<rows, 256, 0, st>>>(p.ccount, p.state, p.nchunks, n_kv_heads, sr);
  sel_hist<0><<<g, 256, 0, st>>>(vals, stride, p.chunk, n_kv_heads, sr, p.hist, p.state);
  sel_scan<0><<<rows, 256, 0, st>>>(p.hist, p.state, n_kv_heads, sr);
  sel_hist<1><<<g, 256, 0, st>>>(vals, stride, p.chunk, n_kv_heads, sr, p.hist, p.state);
  sel_scan<1><<<rows, 256, 0, st>>>(p.hist, p.state, n_kv_heads, sr);
  sel_hist<2><<<g, 256, 0, st>>>(vals, stride, p.chunk, n_kv_heads, sr, p.hist, p.state);
  sel_scan<2><<<rows, 256, 0, st>>>(p.hist, p.state, n_kv_heads, sr);
  sel_count<false><<<g, 256, 0, st>>>(vals, stride, p.chunk, n_kv_heads, sr, p.state, p.ccount);
  sel_offsets<<<rows, 256, 0, st>>>(p.ccount, p.coff, p.nchunks, n_kv_heads, sr);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

// ---------------------------------------------------------------------------------------
// Top-k fast path: one 12-bit histogram pass finds the bin b* that holds the k-th largest key;
// a second pass counts, per chunk, the slots above that bin and collects the (few) slots inside
// it as (key, slot) candidates; one workgroup per row then finishes the radix select on the
// candidates only and turns the counts into chunk offsets for the ordered emit.
constexpr int kBins12 = 4096;
constexpr int kMaxChunks = 1024;

struct TopkWs {
  uint32_t* hist;      // [rows][4096]
  uint32_t* ncand;     // [rows][1024] entries in each chunk's list
  uint32_t* state;     // [rows][4]: T (after resolve), r_eq / still-to-take, b*, unused
  uint32_t* above;     // [rows][1024] slots strictly above bin b* per chunk
  uint32_t* coff;      // [rows][1024][2]
  uint2* cand;         // [rows][row_entries]: chunk c owns entries [c*chunk, (c+1)*chunk)
  int64_t row_entries;
  // cumulative-weight selection only
  uint32_t* pcount;    // [rows][4096] slots per 12-bit bin
  uint64_t* pmass;     // [rows][4096] integer weight per bin
  uint64_t* pstate;    // [rows][4]: target still to reach, Theta, Z, (unused)
  uint32_t* prow;      // [rows][4]: key of the row maximum, slots still allowed, selected count, (unused)
  // scan + top-k in one call only
  uint32_t* samples;   // [rows][kSampleMax] keys of the sampled slots
  uint32_t* spec;      // [rows][4]: threshold key, 1 = row scanned a second time, unused, unused
  uint32_t* mon;       // [rows][4] since the last reset: fused selections, fewest and most pairs a first scan let
                       // through, selections that needed the second scan
};

// chunk geometry for a row of n slots: at most 1024 chunks, each a multiple of 1024 slots, >= 4096
static void chunk_geometry(int64_t n, int64_t* chunk, int32_t* nchunks) {
  if (n < 1) n = 1;
  int64_t c = align_up((n + 1023) / 1024, 1024);
  if (c < 4096) c = 4096;
  *chunk = c;
  *nchunks = (int32_t)((n + c - 1) / c);
}

static int64_t list_entries_per_row(int64_t cap) {
  int64_t chunk;
  int32_t nchunks;
  chunk_geometry(cap, &chunk, &nchunks);
  return align_up(cap, 1024) + 2 * chunk;     // nchunks(n) * chunk(n) < n + chunk(n) <= this, for any n <= cap
}

size_t topk_workspace_bytes(int rows, int64_t cap) {
  size_t b = 0;
  b += align_up((int64_t)rows * kBins12 * 4, 256);
  b += align_up((int64_t)rows * kMaxChunks * 4, 256);
  b += align_up((int64_t)rows * 4 * 4, 256);
  b += align_up((int64_t)rows * 1024 * 4, 256);
  b += align_up((int64_t)rows * 1024 * 2 * 4, 256);
  b += align_up((int64_t)rows * list_entries_per_row(cap) * 8, 256);
  b += align_up((int64_t)rows * kBins12 * 4, 256);
  b += align_up((int64_t)rows * kBins12 * 8, 256);
  b += align_up((int64_t)rows * 4 * 8, 256);
  b += align_up((int64_t)rows * 4 * 4, 256);
  b += align_up((int64_t)rows * kSampleMax * 4, 256);
  b += align_up((int64_t)rows * 4 * 4, 256);
  b += align_up((int64_t)rows * 4 * 4, 256);
  return b;
}

static void topk_carve(TopkWs* t, void* ws, int rows, int64_t cap) {
  uint8_t* w = (uint8_t*)ws;
  t->hist = (uint32_t*)w;  w += align_up((int64_t)rows * kBins12 * 4, 256);
  t->ncand = (uint32_t*)w; w += align_up((int64_t)rows * kMaxChunks * 4, 256);
  t->state = (uint32_t*)w; w += align_up((int64_t)rows * 4 * 4, 256);
  t->above = (uint32_t*)w; w += align_up((int64_t)rows * 1024 * 4, 256);
  t->coff = (uint32_t*)w;  w += align_up((int64_t)rows * 1024 * 2 * 4, 256);
  t->cand = (uint2*)w;
  t->row_entries = list_entries_per_row(cap);
  w += align_up((int64_t)rows * t->row_entries * 8, 256);
  t->pcount = (uint32_t*)w; w += align_up((int64_t)rows * kBins12 * 4, 256);
  t->pmass = (uint64_t*)w;  w += align_up((int64_t)rows * kBins12 * 8, 256);
  t->pstate = (uint64_t*)w; w += align_up((int64_t)rows * 4 * 8, 256);
  t->prow = (uint32_t*)w;   w += align_up((int64_t)rows * 4 * 4, 256);
  t->samples = (uint32_t*)w; w += align_up((int64_t)rows * kSampleMax * 4, 256);
  t->spec = (uint32_t*)w;    w += align_up((int64_t)rows * 4 * 4, 256);
  t->mon = (uint32_t*)w;
}

__global__ void tk_zero(uint32_t* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

// exclusive prefix sum of one value per thread over a 256-thread workgroup
__device__ __forceinline__ uint32_t block_scan_excl_256(uint32_t v, uint32_t* wsum /*[4]*/) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  uint32_t inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t a = __shfl_up(inc, o);
    if (lane >= o) inc += a;
  }
  if (lane == 63) wsum[w] = inc;
  __syncthreads();
  uint32_t base = 0;
  for (int x = 0; x < w; ++x) base += wsum[x];
  __syncthreads();
  return base + inc - v;
}

// LDS counter updates, to be called by all lanes of a wave together.  When every participating lane
// targets the same counter (ties, clustered scores) the wave issues one atomic instead of up to 64
// serialised ones on the same word.
__device__ __forceinline__ void lds_count(uint32_t* h, uint32_t bin, bool hit, bool aggregate) {
  if (!aggregate) {                       // wave-uniform choice: short candidate sets do not pay for the ballots
    if (hit) atomicAdd(&h[bin], 1u);
    return;
  }
  const uint64_t m = __ballot(hit);
  if (m == 0) return;
  const int leader = __ffsll((unsigned long long)m) - 1;
  const uint32_t b0 = __shfl(bin, leader);
  if (__ballot(hit && bin != b0) == 0) {
    if ((int)(threadIdx.x & 63) == leader) atomicAdd(&h[b0], (uint32_t)__popcll(m));
  } else if (hit) {
    atomicAdd(&h[bin], 1u);
  }
}

// The same for a counter and an integer weight; one pair of atomics when all participating lanes hold the
// same key (and therefore the same weight).
__device__ __forceinline__ void lds_count_mass(uint32_t* h, unsigned long long* hm, uint32_t bin, uint32_t key,
                                               uint64_t w, bool hit, bool aggregate) {
  if (!aggregate) {
    if (hit) {
      atomicAdd(&h[bin], 1u);
      if (w) atomicAdd(&hm[bin], (unsigned long long)w);
    }
    return;
  }
  const uint64_t m = __ballot(hit);
  if (m == 0) return;
  const int leader = __ffsll((unsigned long long)m) - 1;
  const uint32_t k0 = __shfl(key, leader);
  if (__ballot(hit && key != k0) == 0) {
    if ((int)(threadIdx.x & 63) == leader) {
      const uint32_t c = (uint32_t)__popcll(m);
      atomicAdd(&h[bin], c);
      if (w) atomicAdd(&hm[bin], (unsigned long long)w * c);
    }
  } else if (hit) {
    atomicAdd(&h[bin], 1u);
    if (w) atomicAdd(&hm[bin], (unsigned long long)w);
  }
}

// Appends the participating lanes' (key, slot) pairs to an LDS list with one counter update per wave.
__device__ __forceinline__ void lds_append(uint32_t* counter, uint2* list, uint32_t room, uint32_t key, uint32_t slot,
                                           bool hit) {
  const uint64_t m = __ballot(hit);
  if (m == 0) return;
  const int lane = threadIdx.x & 63;
  const int leader = __ffsll((unsigned long long)m) - 1;
  uint32_t base = 0;
  if (lane == leader) base = atomicAdd(counter, (uint32_t)__popcll(m));
  base = __shfl(base, leader);
  if (hit) {
    const uint32_t at = base + (uint32_t)__popcll(m & ((1ull << lane) - 1));
    if (at < room) list[at] = uint2{key, slot};
  }
}

// Keys of the 16 slots s0 + x*256 + tid (x = 0..15) of a 4096-slot tile, all loads issued before
// any use; slots at or past `end` yield valid[x] = false.
__device__ __forceinline__ void load_tile_keys(const float* __restrict__ v, int64_t s0, int64_t end,
                                               uint32_t (&key)[16], bool (&valid)[16]) {
  float f[16];
#pragma unroll
  for (int x = 0; x < 16; ++x) {
    const int64_t j = s0 + x * 256 + threadIdx.x;
    valid[x] = j < end;
    f[x] = v[valid[x] ? j : end - 1];
  }
#pragma unroll
  for (int x = 0; x < 16; ++x) key[x] = order_key(f[x]);
}

// 12-bit histogram of a row's keys.
__global__ __launch_bounds__(256) void tk_hist(const float* __restrict__ vals, int64_t stride, int64_t chunk,
                                               int n_kv_heads, SelRows sr, TopkWs t) {
  __shared__ uint32_t lh[kBins12];
  const int row = blockIdx.y;
  const int64_t want = sr.want[row / n_kv_heads];
  if (want <= 0) return;
  const int64_t nsel = sr.nsel[row / n_kv_heads];
  const int64_t c0 = (int64_t)blockIdx.x * chunk;
  if (c0 >= nsel) return;
  int64_t c1 = c0 + chunk;
  if (c1 > nsel) c1 = nsel;
  for (int i = threadIdx.x; i < kBins12; i += 256) lh[i] = 0;
  __syncthreads();
  const float* v = vals + (int64_t)row * stride;
  for (int64_t s0 = c0; s0 < c1; s0 += 4096) {
    uint32_t key[16];
    bool valid[16];
    load_tile_keys(v, s0, c1, key, valid);
#pragma unroll
    for (int x = 0; x < 16; ++x)
      if (valid[x]) atomicAdd(&lh[key[x] >> 20], 1u);
  }
  __syncthreads();
  uint32_t* gh = t.hist + (int64_t)row * kBins12;
  for (int i = threadIdx.x; i < kBins12; i += 256) {
    const uint32_t c = lh[i];
    if (c) atomicAdd(&gh[i], c);
  }
}

// One workgroup per row: locates the bin b* of the `want`-th largest key (bins scanned from the
// top) and leaves (still-to-take, b*, too-many-candidates flag) in state.
__global__ __launch_bounds__(256) void tk_findbin(int n_kv_heads, SelRows sr, TopkWs t) {
  __shared__ uint32_t wsum[4];
  const int row = blockIdx.x;
  const int64_t want = sr.want[row / n_kv_heads];
  if (want <= 0) return;
  uint32_t* gh = t.hist + (int64_t)row * kBins12;
  uint32_t h[16], sum = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int b = kBins12 - 1 - (16 * threadIdx.x + i);
    h[i] = gh[b];
    gh[b] = 0;                 // leave the histogram clean for the next selection on this workspace
    sum += h[i];
  }
  uint32_t running = block_scan_excl_256(sum, wsum);
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    if (running < (uint32_t)want && (uint32_t)want <= running + h[i]) {
      t.state[4 * row + 1] = (uint32_t)want - running;                 // still to take inside the bin
      t.state[4 * row + 2] = kBins12 - 1 - (16 * threadIdx.x + i);     // b*
    }
    running += h[i];
  }
}

// Second pass over the row.  Every chunk writes, in slot order, the (key, slot) pairs of its slots
// in bin b* or above into its own list (room for the whole chunk, so it cannot overflow), and
// counts the ones strictly above the bin.  Lists are per chunk so that no two workgroups ever
// contend for an append position.
__global__ __launch_bounds__(256) void tk_collect(const float* __restrict__ vals, int64_t stride, int64_t chunk,
                                                  int n_kv_heads, SelRows sr, TopkWs t) {
  __shared__ uint32_t wsum[4];
  __shared__ uint32_t pc[64], po[64];
  __shared__ uint32_t s_total;
  const int row = blockIdx.y;
  const int64_t want = sr.want[row / n_kv_heads];
  if (want <= 0) return;
  const int64_t nsel = sr.nsel[row / n_kv_heads];
  const int64_t c0 = (int64_t)blockIdx.x * chunk;
  const uint32_t bin = t.state[4 * row + 2];
  uint32_t* ncand = t.ncand + (int64_t)row * kMaxChunks + blockIdx.x;
  if (c0 >= nsel) {
    if (threadIdx.x == 0) { t.above[(int64_t)row * 1024 + blockIdx.x] = 0; *ncand = 0; }
    return;
  }
  int64_t c1 = c0 + chunk;
  if (c1 > nsel) c1 = nsel;
  const float* v = vals + (int64_t)row * stride;
  uint2* dst = t.cand + (int64_t)row * t.row_entries + (int64_t)blockIdx.x * chunk;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  uint32_t cnt = 0, base = 0;
  for (int64_t s0 = c0; s0 < c1; s0 += 4096) {
    uint32_t key[16];
    bool valid[16];
    load_tile_keys(v, s0, c1, key, valid);
    // slot order inside the tile is (x, wave, lane): one ballot per (x, wave), prefix over the 64 of them
    uint64_t mask[16];
#pragma unroll
    for (int x = 0; x < 16; ++x) {
      const uint32_t b = key[x] >> 20;
      cnt += valid[x] && b > bin;
      mask[x] = __ballot(valid[x] && b >= bin);
      if (lane == 0) pc[x * 4 + w] = (uint32_t)__popcll(mask[x]);
    }
    __syncthreads();
    if (w == 0) {
      const uint32_t mine = pc[lane];
      uint32_t inc = mine;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const uint32_t a2 = __shfl_up(inc, o);
        if (lane >= o) inc += a2;
      }
      po[lane] = inc - mine;
      if (lane == 63) s_total = inc;
    }
    __syncthreads();
#pragma unroll
    for (int x = 0; x < 16; ++x) {
      if ((mask[x] >> lane) & 1) {
        const uint32_t at = base + po[x * 4 + w] + (uint32_t)__popcll(mask[x] & ((1ull << lane) - 1));
        dst[at] = uint2{key[x], (uint32_t)(s0 + x * 256 + threadIdx.x)};
      }
    }
    base += s_total;
    __syncthreads();
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) cnt += __shfl_xor(cnt, o);
  if (lane == 0) wsum[w] = cnt;
  __syncthreads();
  if (threadIdx.x == 0) {
    t.above[(int64_t)row * 1024 + blockIdx.x] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
    *ncand = base;
  }
}

// exclusive prefix sum of one value per thread over a 1024-thread workgroup
__device__ __forceinline__ uint32_t block_scan_excl_1024(uint32_t v, uint32_t* wsum /*[16]*/) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  uint32_t inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t a = __shfl_up(inc, o);
    if (lane >= o) inc += a;
  }
  if (lane == 63) wsum[w] = inc;
  __syncthreads();
  uint32_t base = 0;
  for (int x = 0; x < w; ++x) base += wsum[x];
  __syncthreads();
  return base + inc - v;
}

// One workgroup per row: finishes the select inside bin b* (two 10-bit passes over the
// candidates, or over the whole row when there were too many to keep) and builds the chunk
// offsets of (#key > T, #key == T) for the ordered emit.
constexpr int kResolveLds = 5120;   // candidates staged in LDS by tk_resolve (40 KiB)

// One workgroup per row: finishes the select inside bin b* (two 10-bit passes over the list
// entries that lie in that bin) and builds the chunk offsets of (#key > T, #key == T) for the
// ordered emit.
__global__ __launch_bounds__(1024) void tk_resolve(int64_t chunk, int nchunks, int n_kv_heads, SelRows sr, TopkWs t) {
  __shared__ uint32_t h[1024], e[1024], cnt[1024], wsum[16];
  __shared__ uint32_t s_prefix, s_rem, s_n;
  __shared__ uint2 lc[kResolveLds];
  const int row = blockIdx.x;
  if (sr.want[row / n_kv_heads] <= 0) return;
  const uint32_t bin = t.state[4 * row + 2];
  const uint2* cand = t.cand + (int64_t)row * t.row_entries;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  uint32_t prefix = bin << 20, rem = t.state[4 * row + 1];
  cnt[tid] = tid < nchunks ? t.ncand[(int64_t)row * kMaxChunks + tid] : 0;
  if (tid == 0) s_n = 0;
  __syncthreads();
  // sweep(f): f(key, slot, hit) over every list entry of the row, hit = the entry exists and lies in bin
  // b*; f is called by all lanes of a wave together.  Each wave takes 16 chunks per step and fetches the
  // first 64 entries of all of them in one batch of loads (most lists are shorter than that), so a step
  // costs one memory round trip; longer lists follow, 8 loads in flight.
  auto sweep = [&](auto&& f) {
    for (int c0 = 0; c0 < nchunks; c0 += 256) {
      uint2 ent[16];
      uint32_t m[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int c = c0 + wv * 16 + u;
        m[u] = c < nchunks ? cnt[c] : 0;
        ent[u] = uint2{0, 0};
        if ((uint32_t)lane < m[u]) ent[u] = cand[(int64_t)c * chunk + lane];
      }
#pragma unroll
      for (int u = 0; u < 16; ++u) f(ent[u].x, ent[u].y, (uint32_t)lane < m[u] && (ent[u].x >> 20) == bin);
#pragma unroll 1
      for (int u = 0; u < 16; ++u) {      // long lists (clustered heavy hitters, mass ties)
        const int c = c0 + wv * 16 + u;
        for (uint32_t i0 = 64 + lane; i0 < m[u] + lane; i0 += 512) {
          uint2 x[8];
#pragma unroll
          for (int v = 0; v < 8; ++v) {
            x[v] = uint2{0, 0};
            if (i0 + 64 * v < m[u]) x[v] = cand[(int64_t)c * chunk + i0 + 64 * v];
          }
#pragma unroll
          for (int v = 0; v < 8; ++v) f(x[v].x, x[v].y, i0 + 64 * v < m[u] && (x[v].x >> 20) == bin);
        }
      }
    }
  };
  // staging: the in-bin entries go to the LDS list; one counter update per wave and batch of loads
  {
    const uint64_t lt = (1ull << lane) - 1;
    auto stage = [&](const uint2* x, const bool* hit, int cntx) {
      uint64_t mk[16];
      uint32_t off[16], tot = 0;
#pragma unroll
      for (int u = 0; u < 16; ++u)
        if (u < cntx) { mk[u] = __ballot(hit[u]); off[u] = tot; tot += (uint32_t)__popcll(mk[u]); }
      if (tot == 0) return;
      uint32_t base = 0;
      if (lane == 0) base = atomicAdd(&s_n, tot);
      base = __shfl(base, 0);
#pragma unroll
      for (int u = 0; u < 16; ++u)
        if (u < cntx && hit[u]) {
          const uint32_t at = base + off[u] + (uint32_t)__popcll(mk[u] & lt);
          if (at < (uint32_t)kResolveLds) lc[at] = x[u];
        }
    };
    for (int c0 = 0; c0 < nchunks; c0 += 256) {
      uint2 ent[16];
      bool hit[16];
      uint32_t m[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int c = c0 + wv * 16 + u;
        m[u] = c < nchunks ? cnt[c] : 0;
        ent[u] = uint2{0, 0};
        if ((uint32_t)lane < m[u]) ent[u] = cand[(int64_t)c * chunk + lane];
      }
#pragma unroll
      for (int u = 0; u < 16; ++u) hit[u] = (uint32_t)lane < m[u] && (ent[u].x >> 20) == bin;
      stage(ent, hit, 16);
#pragma unroll 1
      for (int u = 0; u < 16; ++u) {
        const int c = c0 + wv * 16 + u;
        for (uint32_t i0 = 64 + lane; i0 < m[u] + lane; i0 += 512) {
          uint2 x[8];
          bool hx[8];
#pragma unroll
          for (int v = 0; v < 8; ++v) {
            x[v] = uint2{0, 0};
            if (i0 + 64 * v < m[u]) x[v] = cand[(int64_t)c * chunk + i0 + 64 * v];
          }
#pragma unroll
          for (int v = 0; v < 8; ++v) hx[v] = i0 + 64 * v < m[u] && (x[v].x >> 20) == bin;
          stage(x, hx, 8);
        }
      }
    }
  }
  __syncthreads();
  const uint32_t nst = s_n;
  const bool staged = nst <= (uint32_t)kResolveLds;
  auto visit = [&](auto&& f) {
    if (staged) {
      for (uint32_t i0 = 0; i0 < nst; i0 += 1024) {
        const bool hit = i0 + tid < nst;
        const uint2 x = lc[hit ? i0 + tid : 0];
        f(x.x, x.y, hit);
      }
    } else {
      sweep(f);
    }
  };
  for (int pass = 0; pass < 2; ++pass) {
    const int shift = pass == 0 ? 10 : 0;
    h[tid] = 0;
    __syncthreads();
    visit([&](uint32_t key, uint32_t, bool hit) {
      lds_count(h, (key >> shift) & 1023u, hit && (key >> (shift + 10)) == (prefix >> (shift + 10)), !staged);
    });
    __syncthreads();
    const uint32_t mine = h[1023 - tid];                    // thread tid owns bin 1023 - tid
    const uint32_t running = block_scan_excl_1024(mine, wsum);
    if (running < rem && rem <= running + mine) {
      s_prefix = prefix | ((uint32_t)(1023 - tid) << shift);
      s_rem = rem - running;
    }
    __syncthreads();
    prefix = s_prefix;
    rem = s_rem;
    __syncthreads();
  }
  const uint32_t T = prefix;
  h[tid] = 0;
  e[tid] = 0;
  __syncthreads();
  visit([&](uint32_t key, uint32_t slot, bool hit) {
    lds_count(h, (uint32_t)(slot / chunk), hit && key > T, !staged);
    lds_count(e, (uint32_t)(slot / chunk), hit && key == T, !staged);
  });
  __syncthreads();
  const uint32_t g = (tid < nchunks) ? t.above[(int64_t)row * 1024 + tid] + h[tid] : 0;
  const uint32_t q = (tid < nchunks) ? e[tid] : 0;
  const uint32_t og = block_scan_excl_1024(g, wsum);
  const uint32_t oe = block_scan_excl_1024(q, wsum);
  if (tid < nchunks) {
    t.coff[((int64_t)row * nchunks + tid) * 2] = og;
    t.coff[((int64_t)row * nchunks + tid) * 2 + 1] = oe;
  }
  if (tid == 0) { t.state[4 * row] = T; t.state[4 * row + 1] = rem; }
}

// Ordered emit from the per-chunk lists (already in slot order): no further pass over the row.
//   selected(j) = key_j > T  or  (key_j == T and #{i < j : key_i == T} < r_eq)
//   position(j) = #{i < j : key_i > T} + min(#{i < j : key_i == T}, r_eq)
__global__ __launch_bounds__(256) void tk_emit_lists(int64_t chunk, int nchunks, int n_kv_heads, SelRows sr, TopkWs t,
                                                     int32_t k, int32_t* __restrict__ idx, int32_t* __restrict__ count,
                                                     bool count_from_state) {
  __shared__ uint32_t wsum[2][4];
  const int row = blockIdx.y;
  const int64_t want = sr.want[row / n_kv_heads];
  if (blockIdx.x == 0 && threadIdx.x == 0)
    count[row] = want > 0 ? (count_from_state ? (int32_t)t.prow[4 * row + 2] : (int32_t)want) : 0;
  if (want <= 0) return;
  const uint32_t m = t.ncand[(int64_t)row * kMaxChunks + blockIdx.x];
  if (m == 0) return;
  const uint32_t T = t.state[4 * row], req = t.state[4 * row + 1];
  uint32_t base_g = t.coff[((int64_t)row * nchunks + blockIdx.x) * 2];
  uint32_t base_e = t.coff[((int64_t)row * nchunks + blockIdx.x) * 2 + 1];
  const uint2* src = t.cand + (int64_t)row * t.row_entries + (int64_t)blockIdx.x * chunk;
  int32_t* out = idx + (int64_t)row * k;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  for (uint32_t p0 = 0; p0 < m; p0 += 512) {
    uint2 en[2];
    bool fg[2], fe[2];
    uint32_t ng = 0, ne = 0;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const uint32_t p = p0 + 2 * threadIdx.x + i;
      en[i] = src[p < m ? p : m - 1];
      fg[i] = p < m && en[i].x > T;
      fe[i] = p < m && en[i].x == T;
      ng += fg[i]; ne += fe[i];
    }
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
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      if (fg[i] || (fe[i] && pe < req)) out[pg + (pe < req ? pe : req)] = (int32_t)en[i].y;
      pg += fg[i]; pe += fe[i];
    }
    base_g += wsum[0][0] + wsum[0][1] + wsum[0][2] + wsum[0][3];
    base_e += wsum[1][0] + wsum[1][1] + wsum[1][2] + wsum[1][3];
    __syncthreads();
  }
}


// ---------------------------------------------------------------------------------------
// Top-k straight from the scan (Sec. 3.2): the selecting scan has left, per chunk and in slot order, the
// (key, slot) pairs at or above the row's sampled threshold.  One workgroup per row strings the chunks' lists
// together (in LDS when they fit) - the result is the row's candidates in ascending slot order -, runs the whole
// radix select (12 + 10 + 10 bits) over it and writes the selected slots in ascending order:
//   selected(j) = key_j > T  or  (key_j == T and #{i < j : key_i == T} < r_eq)
//   position(j) = #{i < j : key_i > T} + min(#{i < j : key_i == T}, r_eq)
// A row with fewer pairs than it has to select is marked for a second scan without threshold; `only_failed`
// launches handle exactly those rows.
constexpr int kFullLds = 16384;     // pairs held in LDS (128 KiB, dynamic)
constexpr int kSearchMax = 65536;   // pairs still addressed by position when they do not fit LDS
constexpr int kSmallLds = 12288;    // pairs the four-wave form of the selection holds in LDS (96 KiB) ...
// ... when the expected list fits: k <= 4096 (the scan lets about 2.7 times k pairs per row through); longer lists
// are read where they lie, and the launch then asks for no dynamic LDS at all
static uint32_t small_stage_cap(int32_t k) { return k <= 4096 ? (uint32_t)kSmallLds : 0u; }

// counter updates when the lanes of a wave share a handful of bins (the leading bits of keys that all lie
// just above one threshold): one atomic per distinct bin for the first few, single updates for the rest
__device__ __forceinline__ void lds_count_few(uint32_t* h, uint32_t bin, bool hit) {
  uint64_t todo = __ballot(hit);
  const int lane = threadIdx.x & 63;
#pragma unroll 1
  for (int it = 0; it < 4 && todo != 0; ++it) {
    const int leader = __ffsll((unsigned long long)todo) - 1;
    const uint32_t b0 = __shfl(bin, leader);
    const uint64_t same = __ballot(hit && bin == b0) & todo;
    if (lane == leader) atomicAdd(&h[b0], (uint32_t)__popcll(same));
    todo &= ~same;
  }
  if ((todo >> lane) & 1) atomicAdd(&h[bin], 1u);
}

// exclusive prefix sum of one value per thread over a workgroup of NT threads
template <int NT>
__device__ __forceinline__ uint32_t block_scan_excl(uint32_t v, uint32_t* wsum /*[NT / 64]*/) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  uint32_t inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t a = __shfl_up(inc, o);
    if (lane >= o) inc += a;
  }
  if (lane == 63) wsum[w] = inc;
  __syncthreads();
  uint32_t base = 0;
  for (int x = 0; x < w; ++x) base += wsum[x];
  __syncthreads();
  return base + inc - v;
}

// NT = 1024: one large workgroup per row with the row's pairs staged in up to 128 KiB of LDS - the quickest form
// when the chip has a compute unit to spare.  NT = 256: four waves, one per SIMD, with at most 128 registers each
// and up to 96 KiB of LDS for the pairs (stage_cap of them; longer lists are read where they lie, in L2): this
// one fits into the room that a single finished workgroup of a key scan leaves on a compute unit, where the large
// form has to wait until a scan launch has drained from a whole unit - beside back-to-back scans that is one
// chance per launch.  Same result.
template <int NT>
__device__ __forceinline__ void tk_resolve_emit_body(const int64_t chunk, const int nchunks, const int64_t want,
                                                     const SelectOut& so, const int32_t k, int32_t* __restrict__ idx,
                                                     int32_t* __restrict__ count, const bool only_failed, const int row,
                                                     const uint32_t stage_cap) {
  constexpr int NW = NT / 64;              // waves
  constexpr int PER = 1024 / NT;           // chunks (and 10-bit bins) per thread
  extern __shared__ uint2 lc[];
  __shared__ uint32_t h[kBins12], off[1025], wsum[16];
  __shared__ uint32_t s_prefix, s_rem, s_cb;
  const int tid = threadIdx.x;
  uint32_t* spec = so.spec + 4 * row;
  if (want <= 0) {
    if (tid == 0 && !only_failed) count[row] = 0;
    return;
  }
  if (only_failed && spec[1] == 0) return;
  // off[c] = pairs in the chunks before c; off[1024] = all of them.  Thread tid owns chunks [PER tid, PER tid + PER)
  {
    uint32_t mine[PER], sum = 0;
#pragma unroll
    for (int x = 0; x < PER; ++x) {
      const int c = tid * PER + x;
      mine[x] = c < nchunks ? so.ncand[(int64_t)row * kSelectMaxChunks + c] : 0;
      sum += mine[x];
    }
    uint32_t before = block_scan_excl<NT>(sum, wsum);
#pragma unroll
    for (int x = 0; x < PER; ++x) { off[tid * PER + x] = before; before += mine[x]; }
    if (tid == NT - 1) off[1024] = before;
  }
  __syncthreads();
  const uint32_t total = off[1024];
  if (!only_failed && tid == 0 && so.mon != nullptr) {      // one workgroup per row and launches in stream order: no atomics
    uint32_t* m = so.mon + 4 * row;
    m[0] += 1;
    m[1] = total < m[1] ? total : m[1];
    m[2] = total > m[2] ? total : m[2];
    if (total < (uint32_t)want) m[3] += 1;
  }
  if (total < (uint32_t)want) {
    // the sampled threshold was too high: scan the row again, with the second threshold if the first scan counted
    // enough slots at or above it, else without one
    uint32_t sum1 = 0;
#pragma unroll
    for (int x = 0; x < PER; ++x) {
      const int c = tid * PER + x;
      sum1 += c < nchunks ? so.n1[(int64_t)row * kSelectMaxChunks + c] : 0;
    }
    const uint32_t before1 = block_scan_excl<NT>(sum1, wsum);
    if (tid == NT - 1) {
      const uint32_t enough = before1 + sum1 >= (uint32_t)want;
      spec[0] = enough && spec[1] == 0 ? spec[2] : 0;       // (a second failure cannot happen: the count is exact)
      spec[1] = 1;
    }
    return;
  }
  const uint2* gl = so.lists + (int64_t)row * so.row_entries;
  const bool staged = total <= stage_cap;                   // stage_cap pairs of dynamic LDS came with the launch
  // beyond the LDS stage: up to kSearchMax pairs are still addressed by their position in slot order (short lists:
  // walking them chunk by chunk would cost a memory round trip per chunk), more than that are walked chunk by chunk
  const bool by_position = total <= (uint32_t)kSearchMax;
  // pair p of the row in slot order: the chunk c with off[c] <= p < off[c + 1], entry p - off[c] of its list
  auto fetch = [&](uint32_t p) {
    uint32_t c = 0;
#pragma unroll
    for (int s = 512; s >= 1; s >>= 1)
      if (off[c + s] <= p) c += s;
    return gl[(int64_t)c * chunk + (p - off[c])];
  };
  const int lane = tid & 63, wv = tid >> 6;
  uint32_t kmax = 0;                                        // largest key this thread has seen
  if (staged) {
    // 16 lanes per chunk: the first 32 pairs of 64 chunks per wave in 32 loads, all in flight together (nearly
    // all lists are shorter than that); longer lists follow.  Wave wv takes chunks 64 (wv + NW rep) .. + 63
    const int sub = lane >> 4, i = lane & 15;
#pragma unroll 1
    for (int rep = 0; rep < 16 / NW; ++rep) {
      const int cb0 = (wv + NW * rep) * 64;
      uint2 x[16], y[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int c = cb0 + j * 4 + sub;
        const uint32_t m = off[c + 1] - off[c];
        x[j] = (uint32_t)i < m ? gl[(int64_t)c * chunk + i] : uint2{0, 0};
        y[j] = (uint32_t)i + 16 < m ? gl[(int64_t)c * chunk + i + 16] : uint2{0, 0};
      }
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        const int c = cb0 + j * 4 + sub;
        const uint32_t o = off[c], m = off[c + 1] - o;
        if ((uint32_t)i < m) { lc[o + i] = x[j]; kmax = x[j].x > kmax ? x[j].x : kmax; }
        if ((uint32_t)i + 16 < m) { lc[o + i + 16] = y[j]; kmax = y[j].x > kmax ? y[j].x : kmax; }
      }
#pragma unroll 1
      for (int j = 0; j < 16; ++j) {
        const int c = cb0 + j * 4 + sub;
        const uint32_t o = off[c], m = off[c + 1] - o;
        for (uint32_t e = 32 + i; e < m; e += 16) {
          const uint2 z = gl[(int64_t)c * chunk + e];
          lc[o + e] = z;
          kmax = z.x > kmax ? z.x : kmax;
        }
      }
    }
  }
  __syncthreads();
  // visit(f): f(key, slot, exists) over every pair of the row, in any order, called by all lanes of a wave
  // together.  By position: strided over the LDS copy (or, unstaged, through fetch, four pairs in flight per
  // thread).  Otherwise the lists where they are: wave w takes chunks w, w + NW, ... and reads each list 1024
  // pairs at a time (sixteen loads in flight per lane).
  auto visit = [&](auto&& f) {
    if (by_position) {
      if (staged) {
        for (uint32_t i0 = 0; i0 < total; i0 += NT) {
          const bool hit = i0 + tid < total;
          const uint2 x = lc[hit ? i0 + tid : 0];
          f(x.x, x.y, hit);
        }
      } else {
        for (uint32_t i0 = 0; i0 < total; i0 += 4 * NT) {
          uint2 x[4];
#pragma unroll
          for (int v = 0; v < 4; ++v) x[v] = fetch(i0 + v * NT + tid < total ? i0 + v * NT + tid : 0);
#pragma unroll
          for (int v = 0; v < 4; ++v) f(x[v].x, x[v].y, i0 + v * NT + tid < total);
        }
      }
    } else {
      for (int c = wv; c < nchunks; c += NW) {
        const uint32_t m = off[c + 1] - off[c];
        const uint2* src = gl + (int64_t)c * chunk;
        for (uint32_t i0 = 0; i0 < m; i0 += 1024) {
          uint2 x[16];
#pragma unroll
          for (int v = 0; v < 16; ++v) x[v] = i0 + v * 64 + lane < m ? src[i0 + v * 64 + lane] : uint2{0, 0};
#pragma unroll
          for (int v = 0; v < 16; ++v) f(x[v].x, x[v].y, i0 + v * 64 + lane < m);
        }
      }
    }
  };
  if (!staged) visit([&](uint32_t key, uint32_t, bool hit) { if (hit && key > kmax) kmax = key; });
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) { const uint32_t v = __shfl_xor(kmax, o); kmax = v > kmax ? v : kmax; }
  if (lane == 0) wsum[wv] = kmax;
  __syncthreads();
  for (int x = 0; x < NW; ++x) kmax = wsum[x] > kmax ? wsum[x] : kmax;
  __syncthreads();
  // Radix select on d = key - base (every key of the list is >= base, the scan's threshold): pd = the leading
  // digits of d found so far, s = the number of bits of d below them; rem = how many are still to take among the
  // pairs whose d starts with pd, cb = how many such pairs there are.  The first level spreads the occupied
  // range of d over 4096 bins, so the counters are not fought over although the keys share their leading bits.
  const uint32_t base = spec[0];
  const uint32_t maxd = kmax - base;
  int sbits = 32 - __clz((int)(maxd | 1)) - 12;             // bits of maxd beyond the 12 of the first level
  if (sbits < 0) sbits = 0;
  uint32_t pd = 0, rem = (uint32_t)want, cb = total;
  {
    for (int i = tid; i < kBins12; i += NT) h[i] = 0;
    __syncthreads();
    visit([&](uint32_t key, uint32_t, bool hit) { lds_count(h, (key - base) >> sbits, hit, !staged); });
    __syncthreads();
    constexpr int BPT = kBins12 / NT;                       // bins per thread, from the top
    uint32_t hb[BPT], sum = 0;
#pragma unroll
    for (int i = 0; i < BPT; ++i) { hb[i] = h[kBins12 - 1 - (BPT * tid + i)]; sum += hb[i]; }
    uint32_t running = block_scan_excl<NT>(sum, wsum);
#pragma unroll
    for (int i = 0; i < BPT; ++i) {
      if (running < rem && rem <= running + hb[i]) {
        s_prefix = (uint32_t)(kBins12 - 1 - (BPT * tid + i));
        s_rem = rem - running;
        s_cb = hb[i];
      }
      running += hb[i];
    }
    __syncthreads();
    pd = s_prefix;
    rem = s_rem;
    cb = s_cb;
    __syncthreads();
  }
  uint32_t T = 0, req = 0;
  while (true) {                                            // every condition below is uniform over the workgroup
    if (sbits == 0) {                                       // d is fully known: the pairs left all hold one key
      T = base + pd;
      req = rem;
      break;
    }
    if (cb <= 1024) {
      // few pairs left: rank them against each other.  sl = their keys; T is the key with fewer than rem keys
      // above it that, together with its equals, reaches rem.
      uint32_t* sl = h;
      if (tid == 0) s_cb = 0;
      __syncthreads();
      visit([&](uint32_t key, uint32_t, bool hit) {
        if (hit && ((key - base) >> sbits) == pd) sl[atomicAdd(&s_cb, 1u)] = key;
      });
      __syncthreads();
      for (uint32_t me = (uint32_t)tid; me < cb; me += NT) {
        const uint32_t ki = sl[me];
        uint32_t gt = 0, eq = 0;
        for (uint32_t j = 0; j < cb; ++j) {
          const uint32_t kj = sl[j];
          gt += kj > ki;
          eq += kj == ki;
        }
        if (gt < rem && rem <= gt + eq) { s_prefix = ki; s_rem = rem - gt; }   // equal keys write equal values
      }
      __syncthreads();
      T = s_prefix;
      req = s_rem;
      break;
    }
    const int ns = sbits > 10 ? sbits - 10 : 0, width = sbits - ns;
    for (int i = tid; i < 1024; i += NT) h[i] = 0;
    __syncthreads();
    visit([&](uint32_t key, uint32_t, bool hit) {
      const uint32_t d = key - base;
      lds_count(h, (d >> ns) & ((1u << width) - 1), hit && (d >> sbits) == pd, !staged);
    });
    __syncthreads();
    uint32_t mine[PER], msum = 0;                           // thread tid owns bins 1023 - (PER tid + x)
#pragma unroll
    for (int x = 0; x < PER; ++x) { mine[x] = h[1023 - (PER * tid + x)]; msum += mine[x]; }
    uint32_t running = block_scan_excl<NT>(msum, wsum);
#pragma unroll
    for (int x = 0; x < PER; ++x) {
      if (running < rem && rem <= running + mine[x]) {
        s_prefix = (pd << width) | (uint32_t)(1023 - (PER * tid + x));
        s_rem = rem - running;
        s_cb = mine[x];
      }
      running += mine[x];
    }
    __syncthreads();
    pd = s_prefix;
    rem = s_rem;
    cb = s_cb;
    sbits = ns;
    __syncthreads();
  }
  int32_t* out = idx + (int64_t)row * k;
  if (tid == 0) count[row] = (int32_t)want;
  if (by_position) {
    // ordered part by position (slot order): thread tid owns the run [tid * E, tid * E + E)
    const uint32_t E = (total + NT - 1) / NT;
    const uint32_t p0 = (uint32_t)tid * E;
    const uint32_t p1 = p0 + E < total ? p0 + E : total;
    uint32_t ng = 0, ne = 0;
    if (staged) {
      for (uint32_t p = p0; p < p1; ++p) {
        const uint32_t key = lc[p].x;
        ng += key > T;
        ne += key == T;
      }
    } else if (p0 < p1) {
      // the run lies in consecutive entries of consecutive chunks' lists: one search for its start, then a walk
      uint32_t c = 0;
#pragma unroll
      for (int s = 512; s >= 1; s >>= 1)
        if (off[c + s] <= p0) c += s;
      uint32_t e = p0 - off[c];
      for (uint32_t p = p0; p < p1; ++p) {
        while (e >= off[c + 1] - off[c]) { ++c; e = 0; }
        const uint32_t key = gl[(int64_t)c * chunk + e].x;
        ng += key > T;
        ne += key == T;
        ++e;
      }
    }
    uint32_t rg = block_scan_excl<NT>(ng, wsum);            // pairs above T on lower slots
    uint32_t re = block_scan_excl<NT>(ne, wsum);            // pairs equal to T on lower slots
    if (staged) {
      for (uint32_t p = p0; p < p1; ++p) {
        const uint2 x = lc[p];
        if (x.x > T) { out[rg + (re < req ? re : req)] = (int32_t)x.y; ++rg; }
        else if (x.x == T) { if (re < req) out[rg + re] = (int32_t)x.y; ++re; }
      }
    } else if (p0 < p1) {
      uint32_t c = 0;
#pragma unroll
      for (int s = 512; s >= 1; s >>= 1)
        if (off[c + s] <= p0) c += s;
      uint32_t e = p0 - off[c];
      for (uint32_t p = p0; p < p1; ++p) {
        while (e >= off[c + 1] - off[c]) { ++c; e = 0; }
        const uint2 x = gl[(int64_t)c * chunk + e];
        if (x.x > T) { out[rg + (re < req ? re : req)] = (int32_t)x.y; ++rg; }
        else if (x.x == T) { if (re < req) out[rg + re] = (int32_t)x.y; ++re; }
        ++e;
      }
    }
    return;
  }
  // ordered part on the lists where they are: per chunk the pairs above / equal to T, a prefix over the chunks,
  // then every wave walks its chunks again, 64 pairs at a time, positions by ballot
  uint32_t* cg = h;            // [1024] pairs above T per chunk -> pairs above T in the chunks before
  uint32_t* ce = h + 1024;     // the same for pairs equal to T
  __syncthreads();
  for (int c = wv; c < 1024; c += NW) {
    uint32_t g = 0, e = 0;
    if (c < nchunks) {
      const uint32_t m = off[c + 1] - off[c];
      const uint2* src = gl + (int64_t)c * chunk;
      for (uint32_t i0 = 0; i0 < m; i0 += 1024) {
        uint32_t key[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) key[v] = i0 + v * 64 + lane < m ? src[i0 + v * 64 + lane].x : 0u;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const bool live = i0 + v * 64 + lane < m;
          g += (uint32_t)__popcll(__ballot(live && key[v] > T));
          e += (uint32_t)__popcll(__ballot(live && key[v] == T));
        }
      }
    }
    if (lane == 0) { cg[c] = g; ce[c] = e; }
  }
  __syncthreads();
  {
    uint32_t g[PER], e[PER], gs = 0, es = 0;
#pragma unroll
    for (int x = 0; x < PER; ++x) { g[x] = cg[PER * tid + x]; e[x] = ce[PER * tid + x]; gs += g[x]; es += e[x]; }
    uint32_t og = block_scan_excl<NT>(gs, wsum);
    uint32_t oe = block_scan_excl<NT>(es, wsum);
#pragma unroll
    for (int x = 0; x < PER; ++x) {
      cg[PER * tid + x] = og;
      ce[PER * tid + x] = oe;
      og += g[x];
      oe += e[x];
    }
  }
  __syncthreads();
  const uint64_t lt = (1ull << lane) - 1;
  for (int c = wv; c < nchunks; c += NW) {
    const uint32_t m = off[c + 1] - off[c];
    const uint2* src = gl + (int64_t)c * chunk;
    uint32_t pg = cg[c], pe = ce[c];
    for (uint32_t i0 = 0; i0 < m; i0 += 512) {
      uint2 xs[8];
#pragma unroll
      for (int v = 0; v < 8; ++v) xs[v] = i0 + v * 64 + lane < m ? src[i0 + v * 64 + lane] : uint2{0, 0};
#pragma unroll
      for (int v = 0; v < 8; ++v) {
        const bool live = i0 + v * 64 + lane < m;
        const uint2 x = xs[v];
        const bool fg = live && x.x > T, fe = live && x.x == T;
        const uint64_t mg = __ballot(fg), me = __ballot(fe);
        const uint32_t gb = pg + (uint32_t)__popcll(mg & lt), eb = pe + (uint32_t)__popcll(me & lt);
        if (fg) out[gb + (eb < req ? eb : req)] = (int32_t)x.y;
        else if (fe && eb < req) out[gb + eb] = (int32_t)x.y;
        pg += (uint32_t)__popcll(mg);
        pe += (uint32_t)__popcll(me);
      }
    }
  }
}

template <int NT>
__global__ __launch_bounds__(NT) void tk_resolve_emit(int64_t chunk, int nchunks, int n_kv_heads, SelRows sr,
                                                      SelectOut so, int32_t k, int32_t* __restrict__ idx,
                                                      int32_t* __restrict__ count, bool only_failed, uint32_t stage_cap) {
  tk_resolve_emit_body<NT>(chunk, nchunks, sr.want[blockIdx.x / n_kv_heads], so, k, idx, count, only_failed,
                           (int)blockIdx.x, stage_cap);
}

// The selections of two layers in one launch (the step driver's paired form): workgroups [0, rows) take the
// first layer, [rows, 2 rows) the second.
struct ResolveSide {
  int64_t chunk;
  int32_t nchunks;
  int64_t want[kMaxBatch];
  SelectOut so;
  int32_t* idx;
  int32_t* count;
};
template <int NT>
__global__ __launch_bounds__(NT) void tk_resolve_emit_pair(ResolveSide a, ResolveSide b, int rows, int n_kv_heads,
                                                           int32_t k, bool only_failed, uint32_t stage_cap) {
  if ((int)blockIdx.x < rows) {
    tk_resolve_emit_body<NT>(a.chunk, a.nchunks, a.want[blockIdx.x / n_kv_heads], a.so, k, a.idx, a.count, only_failed,
                             (int)blockIdx.x, stage_cap);
  } else {
    const int row = (int)blockIdx.x - rows;
    tk_resolve_emit_body<NT>(b.chunk, b.nchunks, b.want[row / n_kv_heads], b.so, k, b.idx, b.count, only_failed, row,
                             stage_cap);
  }
}

namespace {
struct FusedPlan {
  SelRows sr;
  SelectOut so;
  TopkWs t;
  int64_t chunk;
  int nchunks;
};
int32_t fused_plan(const Layout& L, const NRes& nr, int64_t nmax, int32_t k, void* ws, FusedPlan* f) {
  for (int b = 0; b < kMaxBatch; ++b) { f->sr.nsel[b] = 0; f->sr.want[b] = -1; }
  for (int b = 0; b < L.batch; ++b) {
    f->sr.nsel[b] = nr.n[b];
    f->sr.want[b] = nr.n[b] < k ? nr.n[b] : k;
    if (f->sr.want[b] == 0) f->sr.want[b] = -1;
  }
  topk_carve(&f->t, ws, L.rows, L.cap);
  const int bpw = select_scan_bpw(L, nmax > 0 ? nmax : 1);
  if (bpw == 0) return HCA_ERR_CAPACITY;
  f->chunk = (int64_t)4 * bpw * L.tpb;
  const int64_t nblocks = (nmax + L.tpb - 1) / L.tpb;
  f->nchunks = (int)((nblocks + 4 * bpw - 1) / (4 * bpw));
  if (f->nchunks < 1) f->nchunks = 1;
  if (f->nchunks > kSelectMaxChunks || (int64_t)f->nchunks * f->chunk > f->t.row_entries) return HCA_ERR_CAPACITY;
  f->so = SelectOut{f->t.spec, f->t.ncand, f->t.above, f->t.cand, f->t.samples, f->t.row_entries, select_sample_count(nmax, k),
                    f->t.mon};
  return HCA_OK;
}
}  // namespace

// The fused selection in three parts, each on any stream ordered after the one before.
// 1. threshold from the sample.  The row lengths may be those before the step's token is appended: slots past
//    them are not sampled, and the estimate does not need the one more slot.
int32_t launch_select_threshold(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax,
                                int32_t k, void* ws, hipStream_t st) {
  FusedPlan f;
  int32_t rc = fused_plan(L, nr, nmax, k, ws, &f);
  if (rc != HCA_OK || nmax == 0) return rc;
  return launch_select_sample(L, kcache, q, nr, k, f.so, st);
}

// The parts of the fused selection as a decode step strings them together on one stream: (a) the sampling alone
// and (b) threshold from the samples + append of the step's key, as launches of their own for the step's first
// layers; (c) the selecting scan of a layer carrying (b) for the next layer and (a) for the one after it (lengths
// before those layers' own appends: the one more slot does not matter to the estimate and is not read).
// (nmax, nmax_before, next_nmax: the longest row at the lengths before the step's append - the sampling of a layer
// and its threshold must agree on the sample count, which depends on it.)
int32_t launch_select_samples(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax,
                              int32_t k, void* ws, hipStream_t st) {
  TopkWs t;
  topk_carve(&t, ws, L.rows, L.cap);
  SelectOut so{t.spec, t.ncand, t.above, t.cand, t.samples, t.row_entries, select_sample_count(nmax, k)};
  return launch_select_sample_scores(L, kcache, q, nr, so, st);
}

int32_t launch_select_threshold_append(const Layout& L, void* kcache, const void* k_new, const NRes& nr_before,
                                       int64_t nmax_before, float* acc, int32_t* pos, const NRes& vrow0, int32_t k,
                                       void* ws, hipStream_t st) {
  TopkWs t;
  topk_carve(&t, ws, L.rows, L.cap);
  SelectOut so{t.spec, t.ncand, t.above, t.cand, t.samples, t.row_entries, select_sample_count(nmax_before, k)};
  return launch_select_rank_append(L, kcache, k_new, nr_before, acc, pos, vrow0, k, so, st);
}

SelectOut select_view(const Layout& L, void* ws, int64_t nmax_before, int32_t k) {
  TopkWs t;
  topk_carve(&t, ws, L.rows, L.cap);
  return SelectOut{t.spec, t.ncand, t.above, t.cand, t.samples, t.row_entries, select_sample_count(nmax_before, k)};
}

int32_t launch_select_scan_step(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax,
                                int32_t k, void* ws, hipStream_t st, uint64_t* stamps, const SelectStepNext& nx) {
  FusedPlan f;
  const int32_t rc = fused_plan(L, nr, nmax, k, ws, &f);
  if (rc != HCA_OK) return rc;
  return launch_select_step(L, kcache, q, nr, nmax, f.so, st, stamps, nx);
}

int32_t launch_select_scan_step_pair(const Layout& L, const void* const kcache[2], const void* const q[2],
                                     const NRes nr[2], const int64_t nmax[2], int32_t k, void* const ws[2], hipStream_t st,
                                     uint64_t* const stamps[2], const SelectStepNext nx[2], hipEvent_t done) {
  SelectOut so[2];
  for (int i = 0; i < 2; ++i) {
    FusedPlan f;
    const int32_t rc = fused_plan(L, nr[i], nmax[i], k, ws[i], &f);
    if (rc != HCA_OK) return rc;
    so[i] = f.so;
  }
  return launch_select_step_pair(L, kcache, q, nr, nmax, so, stamps, nx, st, done);
}

// 2. the selecting scan
int32_t launch_select_begin(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax, int32_t k,
                            void* ws, hipStream_t st, uint64_t* stamps) {
  FusedPlan f;
  int32_t rc = fused_plan(L, nr, nmax, k, ws, &f);
  if (rc != HCA_OK || nmax == 0) return rc;
  return launch_select_scan(L, kcache, q, nr, nmax, f.so, false, st, stamps);
}

// 3. the selection over the lists, then,
// for rows whose sampled threshold left too few pairs, a scan with every slot a candidate and the selection
// again (both launches return at once for every other row).
int32_t launch_select_finish(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax, int32_t k,
                             int32_t* idx, int32_t* count, void* ws, hipStream_t st, bool small_wg) {
  FusedPlan f;
  int32_t rc = fused_plan(L, nr, nmax, k, ws, &f);
  if (rc != HCA_OK) return rc;
  if (small_wg) {
    const uint32_t cap = small_stage_cap(k);
    static std::atomic<uint64_t> opted_s{0};
    if (cap * 8 > 64 * 1024) {
      rc = lds_opt_in(reinterpret_cast<const void*>(&tk_resolve_emit<256>), kSmallLds * 8, &opted_s);
      if (rc != HCA_OK) return rc;
    }
    tk_resolve_emit<256><<<L.rows, 256, cap * 8, st>>>(f.chunk, f.nchunks, L.n_kv_heads, f.sr, f.so, k, idx, count, false, cap);
    if (nmax > 0) {
      rc = launch_select_scan(L, kcache, q, nr, nmax, f.so, true, st);
      if (rc != HCA_OK) return rc;
      tk_resolve_emit<256><<<L.rows, 256, 0, st>>>(f.chunk, f.nchunks, L.n_kv_heads, f.sr, f.so, k, idx, count, true, 0u);
    }
    HCA_HIP(hipGetLastError());
    return HCA_OK;
  }
  static std::atomic<uint64_t> opted{0};
  rc = lds_opt_in(reinterpret_cast<const void*>(&tk_resolve_emit<1024>), kFullLds * 8, &opted);
  if (rc != HCA_OK) return rc;
  tk_resolve_emit<1024><<<L.rows, 1024, kFullLds * 8, st>>>(f.chunk, f.nchunks, L.n_kv_heads, f.sr, f.so, k, idx, count, false,
                                                            (uint32_t)kFullLds);
  if (nmax > 0) {
    rc = launch_select_scan(L, kcache, q, nr, nmax, f.so, true, st);
    if (rc != HCA_OK) return rc;
    tk_resolve_emit<1024><<<L.rows, 1024, kFullLds * 8, st>>>(f.chunk, f.nchunks, L.n_kv_heads, f.sr, f.so, k, idx, count, true,
                                                              (uint32_t)kFullLds);
  }
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

// The same for the two layers of a paired scan launch: three launches for the two of them.
int32_t launch_select_finish_pair(const Layout& L, const void* const kcache[2], const void* const q[2], const NRes nr[2],
                                  const int64_t nmax[2], int32_t k, int32_t* const idx[2], int32_t* const count[2],
                                  void* const ws[2], hipStream_t st, bool small_wg) {
  FusedPlan f[2];
  ResolveSide rs[2];
  for (int i = 0; i < 2; ++i) {
    const int32_t rc = fused_plan(L, nr[i], nmax[i], k, ws[i], &f[i]);
    if (rc != HCA_OK) return rc;
    rs[i].chunk = f[i].chunk;
    rs[i].nchunks = f[i].nchunks;
    for (int b = 0; b < kMaxBatch; ++b) rs[i].want[b] = f[i].sr.want[b];
    rs[i].so = f[i].so;
    rs[i].idx = idx[i];
    rs[i].count = count[i];
  }
  int32_t rc = HCA_OK;
  if (small_wg) {
    const uint32_t cap = small_stage_cap(k);
    static std::atomic<uint64_t> opted_s{0};
    if (cap * 8 > 64 * 1024) {
      rc = lds_opt_in(reinterpret_cast<const void*>(&tk_resolve_emit_pair<256>), kSmallLds * 8, &opted_s);
      if (rc != HCA_OK) return rc;
    }
    tk_resolve_emit_pair<256><<<2 * L.rows, 256, cap * 8, st>>>(rs[0], rs[1], L.rows, L.n_kv_heads, k, false, cap);
  } else {
    static std::atomic<uint64_t> opted{0};
    rc = lds_opt_in(reinterpret_cast<const void*>(&tk_resolve_emit_pair<1024>), kFullLds * 8, &opted);
    if (rc != HCA_OK) return rc;
    tk_resolve_emit_pair<1024><<<2 * L.rows, 1024, kFullLds * 8, st>>>(rs[0], rs[1], L.rows, L.n_kv_heads, k, false,
                                                                       (uint32_t)kFullLds);
  }
  if (nmax[0] > 0 && nmax[1] > 0) {
    const SelectOut so2[2] = {f[0].so, f[1].so};
    rc = launch_select_rescan_pair(L, kcache, q, nr, nmax, so2, st);
    if (rc != HCA_OK) return rc;
    // the selection for rows that had to be scanned again - almost never any - in the four-wave form without an
    // LDS stage: beside a running scan the 1024-thread form would wait for a compute unit to drain just to find
    // that it has nothing to do
    tk_resolve_emit_pair<256><<<2 * L.rows, 256, 0, st>>>(rs[0], rs[1], L.rows, L.n_kv_heads, k, true, 0u);
  }
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

int32_t launch_score_topk(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax, int32_t k,
                          int32_t* idx, int32_t* count, void* ws, hipStream_t st) {
  int32_t rc = launch_select_threshold(L, kcache, q, nr, nmax, k, ws, st);
  if (rc != HCA_OK) return rc;
  rc = launch_select_begin(L, kcache, q, nr, nmax, k, ws, st, nullptr);
  if (rc != HCA_OK) return rc;
  return launch_select_finish(L, kcache, q, nr, nmax, k, idx, count, ws, st, tuning().select_wg == 256);
}

// What the last fused selection on this workspace did, per row: pairs that passed the threshold of the scan that
// produced the result, and whether that scan was the second, unthresholded one.
__global__ __launch_bounds__(256) void tk_select_report(TopkWs t, int nchunks, int32_t* __restrict__ candidates,
                                                        int32_t* __restrict__ rescanned) {
  __shared__ uint32_t wsum[4];
  const int row = blockIdx.x;
  uint32_t v = 0;
  for (int c = threadIdx.x; c < nchunks; c += 256) v += t.ncand[(int64_t)row * kMaxChunks + c];
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = v;
  __syncthreads();
  if (threadIdx.x == 0) {
    candidates[row] = (int32_t)(wsum[0] + wsum[1] + wsum[2] + wsum[3]);
    rescanned[row] = (int32_t)t.spec[4 * row + 1];
  }
}

int32_t launch_select_report(const Layout& L, const NRes& nr, int64_t nmax, void* ws, int32_t* candidates,
                             int32_t* rescanned, hipStream_t st) {
  FusedPlan f;
  const int32_t rc = fused_plan(L, nr, nmax, 1, ws, &f);
  if (rc != HCA_OK) return rc;
  tk_select_report<<<L.rows, 256, 0, st>>>(f.t, nmax > 0 ? f.nchunks : 0, candidates, rescanned);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

// The running figures of the fused selections on a workspace (mon above), copied out and / or started afresh.
__global__ void tk_select_monitor(uint32_t* __restrict__ mon, int rows, int32_t* __restrict__ out, int reset) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * 4) return;
  if (out != nullptr) out[i] = (int32_t)mon[i];
  if (reset) mon[i] = (i & 3) == 1 ? 0x7fffffffu : 0u;
}

int32_t launch_select_monitor(const Layout& L, void* ws, int32_t* out, int reset, hipStream_t st) {
  TopkWs t;
  topk_carve(&t, ws, L.rows, L.cap);
  tk_select_monitor<<<(L.rows * 4 + 255) / 256, 256, 0, st>>>(t.mon, L.rows, out, reset);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

// ---------------------------------------------------------------------------------------
// Cumulative-weight selection (Sec. 3.2, Eq. 4): the shortest prefix of the descending order whose
// softmax weight reaches tau.  Weights are integers (fixed-order fp32 arithmetic, see tp_weight), so
// the histogram sums below are exact and independent of the order in which atomics land.  The
// radix walk is the top-k one with two running totals: it stops in the first bin / digit / equal-key
// group where the weight reaches the target or the slot count reaches k_max.
__device__ __forceinline__ float key_to_float(uint32_t key) {
  return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}

// Integer weight of a logit u <= 0 relative to the row maximum: about exp(u) * 2^31.
//   t = u * log2(e); below -64 -> 0; fl = floor(t); f = t - fl in [0, 1) (exact);
//   p = 2^f by a degree-6 polynomial in Horner form with fused multiply-adds, c_k = (ln 2)^k / k!;
//   mant = (uint64)(p * 2^31) (truncated); w = mant >> -fl.
__device__ __forceinline__ uint64_t tp_weight(float u) {
  const float t = u * 1.44269504f;
  if (!(t >= -64.0f)) return 0;
  const float fl = floorf(t);
  const float f = t - fl;
  float p = 1.5403530e-4f;
  p = fmaf(p, f, 1.3333558e-3f);
  p = fmaf(p, f, 9.6181291e-3f);
  p = fmaf(p, f, 5.5504109e-2f);
  p = fmaf(p, f, 2.4022651e-1f);
  p = fmaf(p, f, 6.9314718e-1f);
  p = fmaf(p, f, 1.0f);
  const uint64_t mant = (uint64_t)(p * 2147483648.0f);
  const int sh = (int)(-fl);
  return sh >= 64 ? 0 : mant >> sh;
}

__global__ void tp_init(TopkWs t, int rows) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < (int64_t)rows * kBins12) { t.pcount[i] = 0; t.pmass[i] = 0; }
  if (i < rows * 4) { t.prow[i] = 0; t.pstate[i] = 0; }
}

// Row maximum of the scores, as an order key.
__global__ __launch_bounds__(256) void tp_rowmax(const float* __restrict__ vals, int64_t stride, int64_t chunk,
                                                 int n_kv_heads, SelRows sr, TopkWs t) {
  __shared__ uint32_t wmax[4];
  const int row = blockIdx.y;
  if (sr.want[row / n_kv_heads] <= 0) return;
  const int64_t nsel = sr.nsel[row / n_kv_heads];
  const int64_t c0 = (int64_t)blockIdx.x * chunk;
  if (c0 >= nsel) return;
  int64_t c1 = c0 + chunk;
  if (c1 > nsel) c1 = nsel;
  const float* v = vals + (int64_t)row * stride;
  uint32_t best = 0;
  for (int64_t s0 = c0; s0 < c1; s0 += 4096) {
    uint32_t key[16];
    bool valid[16];
    load_tile_keys(v, s0, c1, key, valid);
#pragma unroll
    for (int x = 0; x < 16; ++x)
      if (valid[x] && key[x] > best) best = key[x];
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const uint32_t other = __shfl_xor(best, o);
    if (other > best) best = other;
  }
  if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = best;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int x = 1; x < 4; ++x) if (wmax[x] > best) best = wmax[x];
    atomicMax(&t.prow[4 * row], best);
  }
}

// 12-bit histogram of slot counts and integer weights.
__global__ __launch_bounds__(256) void tp_hist(const float* __restrict__ vals, int64_t stride, int64_t chunk,
                                               int n_kv_heads, SelRows sr, float sm_scale, TopkWs t) {
  __shared__ uint32_t lc[kBins12];
  __shared__ unsigned long long lm[kBins12];
  const int row = blockIdx.y;
  if (sr.want[row / n_kv_heads] <= 0) return;
  const int64_t nsel = sr.nsel[row / n_kv_heads];
  const int64_t c0 = (int64_t)blockIdx.x * chunk;
  if (c0 >= nsel) return;
  int64_t c1 = c0 + chunk;
  if (c1 > nsel) c1 = nsel;
  for (int i = threadIdx.x; i < kBins12; i += 256) { lc[i] = 0; lm[i] = 0; }
  __syncthreads();
  const float m = key_to_float(t.prow[4 * row]) * sm_scale;
  const float* v = vals + (int64_t)row * stride;
  for (int64_t s0 = c0; s0 < c1; s0 += 4096) {
    uint32_t key[16];
    bool valid[16];
    load_tile_keys(v, s0, c1, key, valid);
#pragma unroll
    for (int x = 0; x < 16; ++x)
      if (valid[x]) {
        const uint64_t w = tp_weight(key_to_float(key[x]) * sm_scale - m);
        atomicAdd(&lc[key[x] >> 20], 1u);
        if (w) atomicAdd(&lm[key[x] >> 20], (unsigned long long)w);
      }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < kBins12; i += 256) {
    const uint32_t c = lc[i];
    if (c) {
      atomicAdd(&t.pcount[(int64_t)row * kBins12 + i], c);
      const unsigned long long mm = lm[i];
      if (mm) atomicAdd(reinterpret_cast<unsigned long long*>(&t.pmass[(int64_t)row * kBins12 + i]), mm);
    }
  }
}

// exclusive prefix sum of one 64-bit value per thread over a 256-thread workgroup; *total gets the sum
__device__ __forceinline__ uint64_t block_scan_excl_256_u64(uint64_t v, uint64_t* wsum /*[4]*/, uint64_t* total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  uint64_t inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint64_t a = __shfl_up((unsigned long long)inc, o);
    if (lane >= o) inc += a;
  }
  if (lane == 63) wsum[w] = inc;
  __syncthreads();
  uint64_t base = 0;
  for (int x = 0; x < w; ++x) base += wsum[x];
  *total = wsum[0] + wsum[1] + wsum[2] + wsum[3];
  __syncthreads();
  return base + inc - v;
}

// One workgroup per row: Z, Theta, and the first bin (from the top) in which the running weight reaches
// Theta or the running count reaches k_max.
__global__ __launch_bounds__(256) void tp_findbin(int n_kv_heads, SelRows sr, uint64_t tau_fix, bool tau_one,
                                                  uint32_t k_max, TopkWs t, uint64_t* __restrict__ mass_out) {
  __shared__ uint64_t wsum64[4];
  __shared__ uint32_t wsum[4];
  const int row = blockIdx.x;
  if (sr.want[row / n_kv_heads] <= 0) {
    if (mass_out != nullptr && threadIdx.x < 2) mass_out[2 * row + threadIdx.x] = 0;
    return;
  }
  uint32_t hc[16], csum = 0;
  uint64_t hm[16], msum = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int b = kBins12 - 1 - (16 * threadIdx.x + i);
    hc[i] = t.pcount[(int64_t)row * kBins12 + b];
    hm[i] = t.pmass[(int64_t)row * kBins12 + b];
    csum += hc[i];
    msum += hm[i];
  }
  uint64_t Z;
  uint64_t run_m = block_scan_excl_256_u64(msum, wsum64, &Z);
  uint32_t run_c = block_scan_excl_256(csum, wsum);
  uint64_t theta = tau_one ? Z : __umul64hi(Z, tau_fix);
  if (theta < 1) theta = 1;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const bool before = run_m < theta && run_c < k_max;
    const bool after = run_m + hm[i] >= theta || run_c + hc[i] >= k_max;
    if (before && after && hc[i] > 0) {
      t.state[4 * row + 2] = kBins12 - 1 - (16 * threadIdx.x + i);   // b*
      t.pstate[4 * row] = theta - run_m;                              // weight still to reach inside the bin
      t.prow[4 * row + 1] = k_max - run_c;                            // slots still allowed
      t.prow[4 * row + 3] = run_c;                                    // slots above the bin
    }
    run_m += hm[i];
    run_c += hc[i];
  }
  if (threadIdx.x == 0) {
    t.pstate[4 * row + 1] = theta;
    t.pstate[4 * row + 2] = Z;
    if (mass_out != nullptr) { mass_out[2 * row] = theta; mass_out[2 * row + 1] = Z; }
  }
}

// exclusive prefix sums over a 1024-thread workgroup (one value per thread)
__device__ __forceinline__ uint64_t block_scan_excl_1024_u64(uint64_t v, uint64_t* wsum /*[16]*/) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  uint64_t inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint64_t a = __shfl_up((unsigned long long)inc, o);
    if (lane >= o) inc += a;
  }
  if (lane == 63) wsum[w] = inc;
  __syncthreads();
  uint64_t base = 0;
  for (int x = 0; x < w; ++x) base += wsum[x];
  __syncthreads();
  return base + inc - v;
}

// One workgroup per row: finishes the walk inside bin b* (two 10-bit digits, then the group of equal
// keys, whose members all weigh the same) and builds the chunk offsets for the ordered emit.
__global__ __launch_bounds__(1024) void tp_resolve(int64_t chunk, int nchunks, int n_kv_heads, SelRows sr, float sm_scale,
                                                   TopkWs t) {
  __shared__ uint32_t h[1024], e[1024], cnt[1024], wsum[16];
  __shared__ unsigned long long hm[1024];
  __shared__ uint64_t wsum64[16];
  __shared__ uint32_t s_prefix, s_krem, s_n;
  __shared__ uint64_t s_mrem;
  __shared__ uint2 lc[kResolveLds];
  const int row = blockIdx.x;
  if (sr.want[row / n_kv_heads] <= 0) return;
  const uint32_t bin = t.state[4 * row + 2];
  const uint2* cand = t.cand + (int64_t)row * t.row_entries;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const float m = key_to_float(t.prow[4 * row]) * sm_scale;
  uint32_t prefix = bin << 20, krem = t.prow[4 * row + 1];
  uint64_t mrem = t.pstate[4 * row];
  cnt[tid] = tid < nchunks ? t.ncand[(int64_t)row * kMaxChunks + tid] : 0;
  if (tid == 0) s_n = 0;
  __syncthreads();
  auto sweep = [&](auto&& f) {
    for (int c0 = 0; c0 < nchunks; c0 += 256) {
#pragma unroll 1
      for (int u = 0; u < 16; ++u) {
        const int c = c0 + wv * 16 + u;
        const uint32_t mu = c < nchunks ? cnt[c] : 0;
        for (uint32_t i0 = lane; i0 < mu + lane; i0 += 512) {
          uint2 x[8];
#pragma unroll
          for (int v = 0; v < 8; ++v) {
            x[v] = uint2{0, 0};
            if (i0 + 64 * v < mu) x[v] = cand[(int64_t)c * chunk + i0 + 64 * v];
          }
#pragma unroll
          for (int v = 0; v < 8; ++v) f(x[v].x, x[v].y, i0 + 64 * v < mu && (x[v].x >> 20) == bin);
        }
      }
    }
  };
  sweep([&](uint32_t key, uint32_t slot, bool hit) { lds_append(&s_n, lc, (uint32_t)kResolveLds, key, slot, hit); });
  __syncthreads();
  const uint32_t nst = s_n;
  const bool staged = nst <= (uint32_t)kResolveLds;
  auto visit = [&](auto&& f) {
    if (staged) {
      for (uint32_t i0 = 0; i0 < nst; i0 += 1024) {
        const bool hit = i0 + tid < nst;
        const uint2 x = lc[hit ? i0 + tid : 0];
        f(x.x, x.y, hit);
      }
    } else {
      sweep(f);
    }
  };
  uint32_t cnt_eq = 0;
  for (int pass = 0; pass < 2; ++pass) {
    const int shift = pass == 0 ? 10 : 0;
    h[tid] = 0;
    hm[tid] = 0;
    __syncthreads();
    visit([&](uint32_t key, uint32_t, bool hit) {
      const bool in = hit && (key >> (shift + 10)) == (prefix >> (shift + 10));
      const uint64_t w = in ? tp_weight(key_to_float(key) * sm_scale - m) : 0;
      lds_count_mass(h, hm, (key >> shift) & 1023u, key, w, in, !staged);
    });
    __syncthreads();
    const uint32_t mine_c = h[1023 - tid];                  // thread tid owns digit 1023 - tid
    const uint64_t mine_m = hm[1023 - tid];
    const uint32_t run_c = block_scan_excl_1024(mine_c, wsum);
    const uint64_t run_m = block_scan_excl_1024_u64(mine_m, wsum64);
    const bool before = run_m < mrem && run_c < krem;
    const bool after = run_m + mine_m >= mrem || run_c + mine_c >= krem;
    if (before && after && mine_c > 0) {
      s_prefix = prefix | ((uint32_t)(1023 - tid) << shift);
      s_mrem = mrem - run_m;
      s_krem = krem - run_c;
    }
    __syncthreads();
    prefix = s_prefix;
    mrem = s_mrem;
    krem = s_krem;
    cnt_eq = h[(prefix >> shift) & 1023u];
    __syncthreads();
  }
  const uint32_t T = prefix;
  // the cnt_eq slots with key == T all weigh w_T: take the least r with r * w_T >= mrem, within the
  // count limit
  const uint64_t wT = tp_weight(key_to_float(T) * sm_scale - m);
  uint64_t need = wT > 0 ? (mrem + wT - 1) / wT : (uint64_t)cnt_eq;
  if (need > krem) need = krem;
  if (need > cnt_eq) need = cnt_eq;
  const uint32_t req = (uint32_t)need;
  h[tid] = 0;
  e[tid] = 0;
  __syncthreads();
  visit([&](uint32_t key, uint32_t slot, bool hit) {
    lds_count(h, (uint32_t)(slot / chunk), hit && key > T, !staged);
    lds_count(e, (uint32_t)(slot / chunk), hit && key == T, !staged);
  });
  __syncthreads();
  const uint32_t g = (tid < nchunks) ? t.above[(int64_t)row * 1024 + tid] + h[tid] : 0;
  const uint32_t q = (tid < nchunks) ? e[tid] : 0;
  const uint32_t og = block_scan_excl_1024(g, wsum);
  const uint32_t oe = block_scan_excl_1024(q, wsum);
  if (tid < nchunks) {
    t.coff[((int64_t)row * nchunks + tid) * 2] = og;
    t.coff[((int64_t)row * nchunks + tid) * 2 + 1] = oe;
  }
  if (tid == nchunks - 1) t.prow[4 * row + 2] = og + g + req;      // selected slots: all above T plus req of the equal ones
  if (tid == 0) { t.state[4 * row] = T; t.state[4 * row + 1] = req; }
}

int32_t launch_topp(const Layout& L, const float* sel, const NRes& nr, int64_t nmax, float sm_scale, double tau,
                    int32_t k_max, int32_t* idx, int32_t* count, uint64_t* mass_opt, void* ws, hipStream_t st) {
  SelRows sr;
  for (int b = 0; b < kMaxBatch; ++b) { sr.nsel[b] = 0; sr.want[b] = -1; }
  for (int b = 0; b < L.batch; ++b) {
    sr.nsel[b] = nr.n[b];
    sr.want[b] = nr.n[b] > 0 ? k_max : -1;
  }
  TopkWs t;
  topk_carve(&t, ws, L.rows, L.cap);
  int64_t chunk;
  int32_t nchunks;
  chunk_geometry(nmax, &chunk, &nchunks);
  dim3 g((unsigned)nchunks, (unsigned)L.rows);
  const bool tau_one = tau >= 1.0;
  const uint64_t tau_fix = tau_one ? 0 : (uint64_t)ldexp(tau, 64);
  if (nmax > 0) {
    const int64_t nz = (int64_t)L.rows * kBins12;
    tp_init<<<(unsigned)((nz + 255) / 256), 256, 0, st>>>(t, L.rows);
    dim3 gh((unsigned)((nchunks + 3) / 4), (unsigned)L.rows);
    tp_rowmax<<<gh, 256, 0, st>>>(sel, L.cap, 4 * chunk, L.n_kv_heads, sr, t);
    tp_hist<<<gh, 256, 0, st>>>(sel, L.cap, 4 * chunk, L.n_kv_heads, sr, sm_scale, t);
    tp_findbin<<<L.rows, 256, 0, st>>>(L.n_kv_heads, sr, tau_fix, tau_one, (uint32_t)k_max, t, mass_opt);
    tk_collect<<<g, 256, 0, st>>>(sel, L.cap, chunk, L.n_kv_heads, sr, t);
    tp_resolve<<<L.rows, 1024, 0, st>>>(chunk, nchunks, L.n_kv_heads, sr, sm_scale, t);
  } else if (mass_opt != nullptr) {
    // no resident slot anywhere: only the per-row (Theta, Z) report has to be cleared
    tp_findbin<<<L.rows, 256, 0, st>>>(L.n_kv_heads, sr, tau_fix, tau_one, (uint32_t)k_max, t, mass_opt);
  }
  tk_emit_lists<<<g, 256, 0, st>>>(chunk, nchunks, L.n_kv_heads, sr, t, k_max, idx, count, true);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

size_t topk_hist_bytes(int rows) { return (size_t)rows * kBins12 * 4; }

int32_t launch_topk(const Layout& L, const float* sel, const NRes& nr, int64_t nmax, int32_t k,
                    int32_t* idx, int32_t* count, void* ws, hipStream_t st, bool hist_clean, int64_t list_cap) {
  SelRows sr;
  for (int b = 0; b < kMaxBatch; ++b) { sr.nsel[b] = 0; sr.want[b] = -1; }
  for (int b = 0; b < L.batch; ++b) {
    sr.nsel[b] = nr.n[b];
    sr.want[b] = nr.n[b] < k ? nr.n[b] : k;
    if (sr.want[b] == 0) sr.want[b] = -1;
  }
  TopkWs t;
  topk_carve(&t, ws, L.rows, list_cap > 0 ? list_cap : L.cap);
  int64_t chunk;
  int32_t nchunks;
  chunk_geometry(nmax, &chunk, &nchunks);
  dim3 g((unsigned)nchunks, (unsigned)L.rows);
  if (nmax > 0) {
    const int64_t nz = (int64_t)L.rows * kBins12;
    // the histogram sits at the start of the workspace; tk_findbin clears what it reads, so a caller
    // that zeroed it once and uses the workspace for nothing else (the step driver) skips this launch
    if (!hist_clean) tk_zero<<<(unsigned)((nz + 255) / 256), 256, 0, st>>>(t.hist, nz);
    // fewer, larger workgroups for the histogram: each flushes its bins with global atomics, and
    // atomics to one address serialise
    dim3 gh((unsigned)((nchunks + 3) / 4), (unsigned)L.rows);
    tk_hist<<<gh, 256, 0, st>>>(sel, L.cap, 4 * chunk, L.n_kv_heads, sr, t);
    tk_findbin<<<L.rows, 256, 0, st>>>(L.n_kv_heads, sr, t);
    tk_collect<<<g, 256, 0, st>>>(sel, L.cap, chunk, L.n_kv_heads, sr, t);
    tk_resolve<<<L.rows, 1024, 0, st>>>(chunk, nchunks, L.n_kv_heads, sr, t);
  }
  tk_emit_lists<<<g, 256, 0, st>>>(chunk, nchunks, L.n_kv_heads, sr, t, k, idx, count, false);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

// What hca_topk itself touches of its workspace when the candidate lists are sized for rows of at most
// `list_cap` slots: everything of topk_carve up to and including the lists.
static size_t topk_only_bytes(int rows, int64_t list_cap) {
  size_t b = 0;
  b += align_up((int64_t)rows * kBins12 * 4, 256);
  b += align_up((int64_t)rows * kMaxChunks * 4, 256);
  b += align_up((int64_t)rows * 4 * 4, 256);
  b += align_up((int64_t)rows * 1024 * 4, 256);
  b += align_up((int64_t)rows * 1024 * 2 * 4, 256);
  b += align_up((int64_t)rows * list_entries_per_row(list_cap) * 8, 256);
  return b;
}

}  // namespace hca

// ---- hca_topk without a workspace argument --------------------------------------------------------------
// The scratch memory of the top-k kernels (histogram, per-chunk counts and offsets, candidate lists) as a
// file-scope device array instead of a caller's workspace, for callers that may not allocate.  Every device the
// library runs on holds its own copy of the array at its own address; in host code the array's name is only a
// handle for hipGetSymbolAddress, never a device address.
constexpr size_t kTopkScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kTopkScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];     // device address of `scratch` on each device, once known

// Address of the current device's copy of `scratch` (looked up on the first call on that device).
int32_t scratch_address(void** out) {
  int dev = 0;
  HCA_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return HCA_ERR_UNSUPPORTED;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    HCA_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (p == nullptr) return hca::hip_fail(hipErrorInvalidSymbol);
    g_scratch_ptr[dev].store(p, std::memory_order_release);      // racing first calls store the same address
  }
  *out = p;
  return HCA_OK;
}
}  // namespace

extern "C" int32_t hca_topk_noalloc(const hca_shape* shape, const float* sel, const int64_t* n_resident, int32_t k,
                                    int32_t* idx, int32_t* count, void* stream) {
  using namespace hca;
  Layout L;
  int32_t rc = make_layout(shape, &L);
  if (rc != HCA_OK) return rc;
  if (sel == nullptr || idx == nullptr || count == nullptr) return HCA_ERR_BAD_ARG;
  if (k < 1 || k > L.cap) return HCA_ERR_CAPACITY;
  NRes nr;
  int64_t nmax;
  rc = load_nres(L, n_resident, &nr, &nmax);
  if (rc != HCA_OK) return rc;
  // the lists are sized for the longest resident row, not for the capacity: the limit is on what is scanned
  const int64_t list_cap = nmax > 0 ? nmax : 1;
  if (topk_only_bytes(L.rows, list_cap) > kTopkScratchBytes) return HCA_ERR_CAPACITY;
  void* ws = nullptr;
  rc = scratch_address(&ws);
  if (rc != HCA_OK) return rc;
  // the array keeps the previous call's contents: launch_topk clears the histogram with a fill kernel
  // (hist_clean = false) and every other region is written before it is read
  return launch_topk(L, sel, nr, nmax, k, idx, count, ws, (hipStream_t)stream, false, list_cap);
}
