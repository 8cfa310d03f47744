// Step 4: accumulated-score eviction with stable compaction.  The keep-set is the newest
// n_protect slots plus the M - n_protect highest accumulated scores among the others (ties
// towards the lower slot); kept slots move to the front in ascending old-slot order.
#include "hca_internal.h"

namespace hca {

struct EvictWs {
  void* select;      // select engine workspace
  int32_t* kept;     // [rows][M] when the caller passes no buffer
  uint8_t* codes;    // [rows][mblk][1024] staging of the compacted code blocks
  uint8_t* meta;     // [rows][mblk][256]
  float* acc;        // [rows][M]
  int32_t* pos;      // [rows][M]
};

// where the compacted rows go: the staging area of the workspace, or a second cache given by the caller
struct EvictDst {
  uint8_t* codes; int64_t codes_row;   // row stride in bytes
  uint8_t* meta;  int64_t meta_row;
  float* acc; int32_t* pos; int64_t ap_row;   // row stride in elements
};

static int64_t mblk_of(const Layout& L, int64_t M) { return (M + L.tpb - 1) / L.tpb; }

size_t evict_workspace_bytes(const Layout& L, int64_t M) {
  const int64_t mb = mblk_of(L, M);
  size_t b = select_workspace_bytes(L.rows, L.cap);
  b += align_up((int64_t)L.rows * M * 4, 256);
  b += align_up((int64_t)L.rows * mb * kBlockBytes, 256);
  b += align_up((int64_t)L.rows * mb * kMetaBytes, 256);
  b += 2 * align_up((int64_t)L.rows * M * 4, 256);
  return b;
}

static void carve(EvictWs* e, void* ws, const Layout& L, int64_t M) {
  const int64_t mb = mblk_of(L, M);
  uint8_t* w = (uint8_t*)ws;
  e->select = w;         w += select_workspace_bytes(L.rows, L.cap);
  e->kept = (int32_t*)w; w += align_up((int64_t)L.rows * M * 4, 256);
  e->codes = w;          w += align_up((int64_t)L.rows * mb * kBlockBytes, 256);
  e->meta = w;           w += align_up((int64_t)L.rows * mb * kMetaBytes, 256);
  e->acc = (float*)w;    w += align_up((int64_t)L.rows * M * 4, 256);
  e->pos = (int32_t*)w;
}

// Ordered pass over all resident slots of a row: writes kept[position] = old slot.
// skip_identity (in-place compaction into the workspace's own list only): a chunk up to whose end every slot is
// kept holds kept[d] = d, which nothing reads - the moves start at the block of the first dropped slot -, so its
// workgroup returns without touching acc or the list.  The chunk prefixes say so: slots kept below the next
// chunk's start = #(above T) + min(#(equal to T), r_eq) counted below it.
__global__ __launch_bounds__(256) void evict_positions(const float* __restrict__ acc, int64_t stride, int64_t chunk,
                                                       int nchunks, int n_kv_heads, SelRows sr, NRes nr,
                                                       uint32_t* __restrict__ state,
                                                       const uint32_t* __restrict__ coff, int64_t M,
                                                       int32_t* __restrict__ kept, int skip_identity) {
  __shared__ uint32_t wsum[2][4];
  const int row = blockIdx.y;
  const int b = row / n_kv_heads;
  const int64_t want = sr.want[b];
  if (want < 0) return;
  const int64_t nsel = sr.nsel[b], n = nr.n[b];
  const int64_t c0 = (int64_t)blockIdx.x * chunk;
  if (c0 >= n) return;
  int64_t c1 = c0 + chunk;
  if (c1 > n) c1 = n;
  const uint32_t T = state[4 * row], req = state[4 * row + 1];
  if (skip_identity && (int)blockIdx.x + 1 < nchunks && c0 + chunk <= nsel) {
    const uint32_t ng = coff[((int64_t)row * nchunks + blockIdx.x + 1) * 2];
    const uint32_t ne = coff[((int64_t)row * nchunks + blockIdx.x + 1) * 2 + 1];
    if ((int64_t)ng + (int64_t)(ne < req ? ne : req) == c0 + chunk) return;
  }
  uint32_t base_g = coff[((int64_t)row * nchunks + blockIdx.x) * 2];
  uint32_t base_e = coff[((int64_t)row * nchunks + blockIdx.x) * 2 + 1];
  const float* v = acc + (int64_t)row * stride;
  int32_t* out = kept + (int64_t)row * M;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  uint32_t hole = 0xffffffffu;               // lowest slot this thread saw dropped
  for (int64_t s0 = c0; s0 < c1; s0 += 1024) {
    const int64_t j0 = s0 + 4 * threadIdx.x;
    bool fg[4], fe[4];
    uint32_t ng = 0, ne = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t j = j0 + i;
      uint32_t key = 0;
      const bool in = j < nsel;
      if (in) key = order_key(v[j]);
      fg[i] = in && key > T;
      fe[i] = in && key == T;
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
    const uint32_t tot_g = wsum[0][0] + wsum[0][1] + wsum[0][2] + wsum[0][3];
    const uint32_t tot_e = wsum[1][0] + wsum[1][1] + wsum[1][2] + wsum[1][3];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t j = j0 + i;
      const bool take = fg[i] || (fe[i] && pe < req);
      if (take) out[pg + (pe < req ? pe : req)] = (int32_t)j;
      else if (j < nsel && (uint32_t)j < hole) hole = (uint32_t)j;
      if (j >= nsel && j < n) out[want + (j - nsel)] = (int32_t)j;  // protected newest slots
      pg += fg[i]; pe += fe[i];
    }
    base_g += tot_g; base_e += tot_e;
    __syncthreads();
  }
  // every slot below the first dropped one keeps its place: the moves can start there
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const uint32_t other = __shfl_xor(hole, o);
    if (other < hole) hole = other;
  }
  if (lane == 0 && hole != 0xffffffffu) atomicMin(&state[4 * row + 2], hole);
}

// kept[d] -> staging slot d.  One thread per (d, j) 16-byte (4-bit) or 8-byte (2-bit) piece.
template <int BITS>
__global__ __launch_bounds__(256) void evict_gather(Layout L, const uint8_t* __restrict__ kcache,
                                                    const float* __restrict__ acc, const int32_t* __restrict__ pos,
                                                    int n_kv_heads, SelRows sr, int64_t M, int64_t d0, int64_t d1,
                                                    const int32_t* __restrict__ kept, EvictDst e,
                                                    const uint32_t* __restrict__ first_hole) {
  const int row = blockIdx.y;
  if (sr.want[row / n_kv_heads] < 0) return;
  // in place: slots below the block of the first dropped slot already hold their own data, so the walk starts
  // there (the grid is modest and strides: when the dropped slots sit near the end, as they do when ties go
  // against the higher slot, almost nothing is launched in vain)
  if (first_hole != nullptr) {
    const int64_t lo = (int64_t)(first_hole[4 * row + 2] & ~(uint32_t)(L.tpb - 1));
    if (lo > d0) d0 = lo;
  }
  const uint8_t* crow = kcache + (int64_t)row * L.codes_row_bytes();
  const uint8_t* mrow = kcache + L.meta_off + (int64_t)row * L.meta_row_bytes();
  uint8_t* cdst = e.codes + (int64_t)row * e.codes_row;
  uint8_t* mdst = e.meta + (int64_t)row * e.meta_row;
  for (int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x; gid < (d1 - d0) * 4; gid += (int64_t)gridDim.x * 256) {
  const int64_t d = d0 + (gid >> 2);
  const int j = (int)(gid & 3);
  const int64_t s = kept[(int64_t)row * M + d];
  if (BITS == 4) {
    const uint4 w = *reinterpret_cast<const uint4*>(crow + (s >> 4) * kBlockBytes + ((s & 15) + 16 * j) * 16);
    *reinterpret_cast<uint4*>(cdst + (d >> 4) * kBlockBytes + ((d & 15) + 16 * j) * 16) = w;
    if (j == 0)
      *reinterpret_cast<uint4*>(mdst + (d >> 4) * kMetaBytes + (d & 15) * 16) =
          *reinterpret_cast<const uint4*>(mrow + (s >> 4) * kMetaBytes + (s & 15) * 16);
  } else {
    const uint2 w = *reinterpret_cast<const uint2*>(crow + (s >> 5) * kBlockBytes + ((s & 15) + 16 * j) * 16 +
                                                    8 * ((s >> 4) & 1));
    *reinterpret_cast<uint2*>(cdst + (d >> 5) * kBlockBytes + ((d & 15) + 16 * j) * 16 + 8 * ((d >> 4) & 1)) = w;
    if (j == 0)
      *reinterpret_cast<uint2*>(mdst + (d >> 5) * kMetaBytes + (d & 31) * 8) =
          *reinterpret_cast<const uint2*>(mrow + (s >> 5) * kMetaBytes + (s & 31) * 8);
  }
  if (j == 1) e.acc[(int64_t)row * e.ap_row + d] = acc[(int64_t)row * L.cap + s];
  if (j == 2) e.pos[(int64_t)row * e.ap_row + d] = pos[(int64_t)row * L.cap + s];
  }
}

// staging -> front of the cache (whole blocks; slots past M in the last block are dead).
__global__ __launch_bounds__(256) void evict_copyback(Layout L, uint8_t* __restrict__ kcache, float* __restrict__ acc,
                                                      int32_t* __restrict__ pos, int n_kv_heads, SelRows sr,
                                                      int64_t M, int64_t mblk, EvictWs e,
                                                      const uint32_t* __restrict__ first_hole) {
  const int row = blockIdx.y;
  if (sr.want[row / n_kv_heads] < 0) return;
  const int64_t d_start = (int64_t)(first_hole[4 * row + 2] & ~(uint32_t)(L.tpb - 1));   // block-aligned
  const int64_t b_start = d_start / L.tpb;
  uint4* cdst = reinterpret_cast<uint4*>(kcache + (int64_t)row * L.codes_row_bytes());
  uint4* mdst = reinterpret_cast<uint4*>(kcache + L.meta_off + (int64_t)row * L.meta_row_bytes());
  const uint4* csrc = reinterpret_cast<const uint4*>(e.codes + (int64_t)row * mblk * kBlockBytes);
  const uint4* msrc = reinterpret_cast<const uint4*>(e.meta + (int64_t)row * mblk * kMetaBytes);
  const int64_t stride = (int64_t)gridDim.x * 256, t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  for (int64_t i = b_start * (kBlockBytes / 16) + t; i < mblk * (kBlockBytes / 16); i += stride) cdst[i] = csrc[i];
  for (int64_t i = b_start * (kMetaBytes / 16) + t; i < mblk * (kMetaBytes / 16); i += stride) mdst[i] = msrc[i];
  for (int64_t i = d_start + t; i < M; i += stride) {
    acc[(int64_t)row * L.cap + i] = e.acc[(int64_t)row * M + i];
    pos[(int64_t)row * L.cap + i] = e.pos[(int64_t)row * M + i];
  }
}

// Out-of-place mode: rows that are not compacted (n <= M) are carried over unchanged.
__global__ __launch_bounds__(256) void evict_carry_rows(Layout L, const uint8_t* __restrict__ src, const float* __restrict__ acc,
                                                        const int32_t* __restrict__ pos, int n_kv_heads, SelRows sr,
                                                        NRes nr, EvictDst e) {
  const int row = blockIdx.y;
  if (sr.want[row / n_kv_heads] >= 0) return;         // compacted rows are written by evict_gather
  const int64_t n = nr.n[row / n_kv_heads];
  const int64_t nblk = (n + L.tpb - 1) / L.tpb;
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const uint4* cs = reinterpret_cast<const uint4*>(src + (int64_t)row * L.codes_row_bytes());
  const uint4* ms = reinterpret_cast<const uint4*>(src + L.meta_off + (int64_t)row * L.meta_row_bytes());
  uint4* cd = reinterpret_cast<uint4*>(e.codes + (int64_t)row * e.codes_row);
  uint4* md = reinterpret_cast<uint4*>(e.meta + (int64_t)row * e.meta_row);
  if (gid < nblk * (kBlockBytes / 16)) cd[gid] = cs[gid];
  if (gid < nblk * (kMetaBytes / 16)) md[gid] = ms[gid];
  if (gid < n) {
    e.acc[(int64_t)row * e.ap_row + gid] = acc[(int64_t)row * L.cap + gid];
    e.pos[(int64_t)row * e.ap_row + gid] = pos[(int64_t)row * L.cap + gid];
  }
}

// Eviction in two host-visible phases so that a step driver can interleave the pieces with other
// work on the same stream: prepare (keep-set selection, positions, carry-over of untouched rows)
// and move (destination slots [d0, d1) of the compaction; d1 == M finishes, with the copy-back
// when the eviction is in place).
struct EvictPlan {
  SelRows sr;
  EvictWs e;
  EvictDst d;
  int32_t* kept;
  uint32_t* state;   // select state: [4 * row + 2] = lowest dropped slot of the row (after evict_positions)
  int64_t M, mblk;
  bool oop, any;
};

static int32_t evict_prepare(const Layout& L, void* kcache, float* acc, int32_t* pos, const NRes& nr, int64_t nmax,
                             int64_t M, int64_t n_protect, int32_t* kept, void* ws, void* kcache_dst,
                             float* acc_dst, int32_t* pos_dst, hipStream_t st, EvictPlan* pl) {
  SelRows& sr = pl->sr;
  pl->any = false;
  for (int b = 0; b < kMaxBatch; ++b) { sr.nsel[b] = 0; sr.want[b] = -1; }
  for (int b = 0; b < L.batch; ++b) {
    if (nr.n[b] > M) {
      sr.nsel[b] = nr.n[b] - n_protect;
      sr.want[b] = M - n_protect;
      pl->any = true;
    }
  }
  pl->oop = kcache_dst != nullptr;
  pl->M = M;
  carve(&pl->e, ws, L, M);
  pl->mblk = mblk_of(L, M);
  EvictDst& d = pl->d;
  if (pl->oop) {
    d.codes = (uint8_t*)kcache_dst;            d.codes_row = L.codes_row_bytes();
    d.meta = (uint8_t*)kcache_dst + L.meta_off; d.meta_row = L.meta_row_bytes();
    d.acc = acc_dst; d.pos = pos_dst; d.ap_row = L.cap;
  } else {
    d.codes = pl->e.codes; d.codes_row = pl->mblk * kBlockBytes;
    d.meta = pl->e.meta;   d.meta_row = pl->mblk * kMetaBytes;
    d.acc = pl->e.acc; d.pos = pl->e.pos; d.ap_row = M;
  }
  bool carry = false;                      // any row that is not compacted?
  for (int b = 0; b < L.batch; ++b) carry = carry || nr.n[b] <= M;
  if (pl->oop && carry && nmax > 0) {
    const int64_t nblk = (nmax + L.tpb - 1) / L.tpb;
    int64_t items = nblk * (kBlockBytes / 16);
    if (items < nmax) items = nmax;
    dim3 gr((unsigned)((items + 255) / 256), (unsigned)L.rows);
    evict_carry_rows<<<gr, 256, 0, st>>>(L, (const uint8_t*)kcache, acc, pos, L.n_kv_heads, sr, nr, d);
  }
  if (!pl->any) {
    if (pl->oop) HCA_HIP(hipGetLastError());
    return HCA_OK;
  }
  pl->kept = kept != nullptr ? kept : pl->e.kept;
  SelectPlan p;
  select_plan(&p, pl->e.select, L.rows, nmax);
  int32_t rc = select_run(p, acc, L.cap, L.rows, L.n_kv_heads, sr, st);
  if (rc != HCA_OK) return rc;
  dim3 g((unsigned)p.nchunks, (unsigned)L.rows);
  pl->state = p.state;
  evict_positions<<<g, 256, 0, st>>>(acc, L.cap, p.chunk, p.nchunks, L.n_kv_heads, sr, nr, p.state, p.coff, M, pl->kept,
                                     (!pl->oop && kept == nullptr) ? 1 : 0);
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

static int32_t evict_move(const Layout& L, void* kcache, float* acc, int32_t* pos, const EvictPlan& pl, int64_t d0,
                          int64_t d1, hipStream_t st) {
  if (!pl.any || d1 <= d0) return HCA_OK;
  // at most 2048 workgroups in all: the kernels stride over what there is to move
  const int64_t cap_wg = L.rows >= 2048 ? 1 : 2048 / L.rows;
  int64_t wg = ((d1 - d0) * 4 + 255) / 256;
  if (wg > cap_wg) wg = cap_wg;
  dim3 gg((unsigned)wg, (unsigned)L.rows);
  if (L.bits == 4)
    evict_gather<4><<<gg, 256, 0, st>>>(L, (const uint8_t*)kcache, acc, pos, L.n_kv_heads, pl.sr, pl.M, d0, d1, pl.kept, pl.d,
                                        pl.oop ? nullptr : pl.state);
  else
    evict_gather<2><<<gg, 256, 0, st>>>(L, (const uint8_t*)kcache, acc, pos, L.n_kv_heads, pl.sr, pl.M, d0, d1, pl.kept, pl.d,
                                        pl.oop ? nullptr : pl.state);
  if (!pl.oop && d1 == pl.M) {
    int64_t items = pl.mblk * (kBlockBytes / 16);
    if (items < pl.M) items = pl.M;
    int64_t wc = (items + 255) / 256;
    if (wc > cap_wg) wc = cap_wg;
    dim3 gc((unsigned)wc, (unsigned)L.rows);
    evict_copyback<<<gc, 256, 0, st>>>(L, (uint8_t*)kcache, acc, pos, L.n_kv_heads, pl.sr, pl.M, pl.mblk, pl.e, pl.state);
  }
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

int32_t launch_evict(const Layout& L, void* kcache, float* acc, int32_t* pos, const NRes& nr, int64_t nmax,
                     int64_t M, int64_t n_protect, int32_t* kept, void* ws, void* kcache_dst, float* acc_dst,
                     int32_t* pos_dst, hipStream_t st) {
  EvictPlan pl;
  int32_t rc = evict_prepare(L, kcache, acc, pos, nr, nmax, M, n_protect, kept, ws, kcache_dst, acc_dst, pos_dst, st, &pl);
  if (rc != HCA_OK) return rc;
  return evict_move(L, kcache, acc, pos, pl, 0, M, st);
}

// out byte p = in byte (p + r) % 16, 0 <= r < 16
__device__ __forceinline__ uint4 rotate_bytes(uint4 x, int r) {
  const uint32_t w[4] = {x.x, x.y, x.z, x.w};
  const int q = r >> 2;
  uint32_t a[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    a[i] = q == 0 ? w[i] : q == 1 ? w[(i + 1) & 3] : q == 2 ? w[(i + 2) & 3] : w[(i + 3) & 3];
  const uint32_t t = (uint32_t)(r & 3);
  uint4 o;
  o.x = __builtin_amdgcn_alignbyte(a[1], a[0], t);
  o.y = __builtin_amdgcn_alignbyte(a[2], a[1], t);
  o.z = __builtin_amdgcn_alignbyte(a[3], a[2], t);
  o.w = __builtin_amdgcn_alignbyte(a[0], a[3], t);
  return o;
}

// ---- codebook caches: the rows that move are index rows of g bytes (or 2 g with 16-bit indices) ----
// A call moves a window of `pieces` 16-byte pieces of every row: source rows of sb bytes, window at piece
// sp0; destination rows of db bytes, window at piece dp0.  acc and pos travel with the call whose source
// window starts at piece 0.
// kept[d] -> destination slot d; one thread per 16-byte piece.  rot: byte indices stored rotated by the slot
// number, re-rotated for the slot they move to.
// Wide form (tiled 16-bit indices): one 16-byte piece = the indices of 8 consecutive groups of a slot, picked
// out of / put back into the group-major tiles; between the two they travel as token-major rows.
__device__ __forceinline__ uint4 vq_wide_read8(const uint16_t* pw, int g, int64_t tiles, int64_t row, int64_t slot, int g0) {
  uint32_t w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
    w[i] = (uint32_t)pw[vq_wide_at(g, tiles, row, slot, g0 + 2 * i)] |
           ((uint32_t)pw[vq_wide_at(g, tiles, row, slot, g0 + 2 * i + 1)] << 16);
  return uint4{w[0], w[1], w[2], w[3]};
}
__device__ __forceinline__ void vq_wide_write8(uint16_t* pw, int g, int64_t tiles, int64_t row, int64_t slot, int g0, uint4 v) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    pw[vq_wide_at(g, tiles, row, slot, g0 + 2 * i)] = (uint16_t)(w[i] & 0xffffu);
    pw[vq_wide_at(g, tiles, row, slot, g0 + 2 * i + 1)] = (uint16_t)(w[i] >> 16);
  }
}

// form: 0 = narrow (byte indices, rotated records), 1 = wide source and destination caches, 2 = wide source cache
// and token-major destination (the staging area)
__global__ __launch_bounds__(256) void vq_evict_gather(int sb, int sp0, int db, int dp0, int pieces, int form, int g,
                                                       int64_t cap, int64_t dcap, const uint8_t* __restrict__ pcache,
                                                       const float* __restrict__ acc, const int32_t* __restrict__ pos,
                                                       int n_kv_heads, SelRows sr, int64_t M,
                                                       const int32_t* __restrict__ kept, uint8_t* __restrict__ pdst,
                                                       float* __restrict__ adst, int32_t* __restrict__ odst,
                                                       int64_t dst_row, const uint32_t* __restrict__ first_hole) {
  const int row = blockIdx.y;
  if (sr.want[row / n_kv_heads] < 0) return;
  // in place: slots below the first dropped one keep their rows, the walk (a modest grid that strides) starts there
  const int64_t lo = first_hole != nullptr ? (int64_t)first_hole[4 * row + 2] : 0;
  for (int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x; gid < (M - lo) * pieces; gid += (int64_t)gridDim.x * 256) {
    const int64_t d = lo + gid / pieces;
    const int j = (int)(gid % pieces);
    const int64_t s = kept[(int64_t)row * M + d];
    if (form == 0) {
      // a rotated record's rotation follows its slot: byte p of slot d is byte (p + d - s) % 16 of slot s
      const uint4 v = reinterpret_cast<const uint4*>(pcache + ((int64_t)row * cap + s) * sb)[sp0 + j];
      reinterpret_cast<uint4*>(pdst + ((int64_t)row * dst_row + d) * db)[dp0 + j] = rotate_bytes(v, (int)((d - s) & 15));
    } else {
      const uint4 v = vq_wide_read8(reinterpret_cast<const uint16_t*>(pcache), g, vq_tiles(cap), row, s, 8 * (sp0 + j));
      if (form == 1) vq_wide_write8(reinterpret_cast<uint16_t*>(pdst), g, vq_tiles(dcap), row, d, 8 * (dp0 + j), v);
      else reinterpret_cast<uint4*>(pdst + ((int64_t)row * dst_row + d) * db)[dp0 + j] = v;
    }
    if (sp0 == 0 && j == 0) adst[(int64_t)row * dst_row + d] = acc[(int64_t)row * cap + s];
    if (sp0 == 0 && (j == 1 || pieces == 1)) odst[(int64_t)row * dst_row + d] = pos[(int64_t)row * cap + s];
  }
}

// Copies a window of the first cnt[b] slots of every row that `which` selects from (src, row stride ssrc
// slots) to (dst, sdst): the copy-back of an in-place eviction (compacted rows, cnt = M) and the carry-over
// of untouched rows of an out-of-place one (cnt = n).  acc and pos go with the call whose destination
// window starts at piece 0.
// first_hole (in-place copy-back only): slots below the row's lowest dropped slot are left alone.
// form: 0 = plain rows on both sides, 1 = wide caches on both sides (carry-over), 2 = token-major source (the
// staging area) into a wide cache (copy-back)
__global__ __launch_bounds__(256) void vq_evict_copy_rows(int sb, int sp0, int db, int dp0, int pieces, int form, int g,
                                                          int64_t scap, int64_t dcap, int n_kv_heads,
                                                          SelRows sr, bool compacted, NRes cnt,
                                                          const uint32_t* __restrict__ first_hole,
                                                          const uint8_t* __restrict__ psrc, const float* __restrict__ asrc,
                                                          const int32_t* __restrict__ osrc, int64_t ssrc,
                                                          uint8_t* __restrict__ pdst, float* __restrict__ adst,
                                                          int32_t* __restrict__ odst, int64_t sdst) {
  const int row = blockIdx.y;
  const int b = row / n_kv_heads;
  if ((sr.want[b] >= 0) != compacted) return;
  const int64_t m = cnt.n[b];
  const int64_t lo = first_hole != nullptr ? (int64_t)first_hole[4 * row + 2] : 0;
  for (int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x; gid < (m - lo) * pieces; gid += (int64_t)gridDim.x * 256) {
    const int64_t d = lo + gid / pieces;
    const int j = (int)(gid % pieces);
    if (form == 0) {
      reinterpret_cast<uint4*>(pdst + ((int64_t)row * sdst + d) * db)[dp0 + j] =
          reinterpret_cast<const uint4*>(psrc + ((int64_t)row * ssrc + d) * sb)[sp0 + j];
    } else {
      const uint4 v = form == 1 ? vq_wide_read8(reinterpret_cast<const uint16_t*>(psrc), g, vq_tiles(scap), row, d, 8 * (sp0 + j))
                                : reinterpret_cast<const uint4*>(psrc + ((int64_t)row * ssrc + d) * sb)[sp0 + j];
      vq_wide_write8(reinterpret_cast<uint16_t*>(pdst), g, vq_tiles(dcap), row, d, 8 * (dp0 + j), v);
    }
    if (dp0 == 0 && j == 0) {
      adst[(int64_t)row * sdst + d] = asrc[(int64_t)row * ssrc + d];
      odst[(int64_t)row * sdst + d] = osrc[(int64_t)row * ssrc + d];
    }
  }
}

int32_t launch_vq_evict(const Layout& L, int g, int c, uint8_t* pcache, float* acc, int32_t* pos, const NRes& nr,
                        int64_t nmax, int64_t M, int64_t n_protect, int32_t* kept, void* ws, uint8_t* pcache_dst,
                        float* acc_dst, int32_t* pos_dst, hipStream_t st) {
  SelRows sr;
  bool any = false, carry = false;
  for (int b = 0; b < kMaxBatch; ++b) { sr.nsel[b] = 0; sr.want[b] = -1; }
  for (int b = 0; b < L.batch; ++b) {
    if (nr.n[b] > M) {
      sr.nsel[b] = nr.n[b] - n_protect;
      sr.want[b] = M - n_protect;
      any = true;
    } else {
      carry = true;
    }
  }
  const bool oop = pcache_dst != nullptr;
  const bool wide = vq_is_wide(L, g, c);
  const int rb = g * (wide ? 2 : 1);        // bytes of an index row: 32 .. 128
  const int pieces = rb / 16;
  EvictWs e;                                // the staging holds 64 bytes per slot (sized for uniform codes)
  carve(&e, ws, L, M);
  const int64_t cap_wg = L.rows >= 2048 ? 1 : 2048 / L.rows;   // at most 2048 workgroups in all: the kernels stride
  auto wgs = [&](int64_t items) { const int64_t w = (items + 255) / 256; return (unsigned)(w > cap_wg ? cap_wg : (w < 1 ? 1 : w)); };
  if (oop && carry && nmax > 0) {
    dim3 gr(wgs(nmax * pieces), (unsigned)L.rows);
    vq_evict_copy_rows<<<gr, 256, 0, st>>>(rb, 0, rb, 0, pieces, wide ? 1 : 0, g, L.cap, L.cap, L.n_kv_heads, sr, false, nr,
                                           nullptr, pcache, acc, pos, L.cap, pcache_dst, acc_dst, pos_dst, L.cap);
  }
  if (!any) {
    if (oop) HCA_HIP(hipGetLastError());
    return HCA_OK;
  }
  int32_t* kp = kept != nullptr ? kept : e.kept;
  SelectPlan p;
  select_plan(&p, e.select, L.rows, nmax);
  int32_t rc = select_run(p, acc, L.cap, L.rows, L.n_kv_heads, sr, st);
  if (rc != HCA_OK) return rc;
  dim3 g1((unsigned)p.nchunks, (unsigned)L.rows);
  evict_positions<<<g1, 256, 0, st>>>(acc, L.cap, p.chunk, p.nchunks, L.n_kv_heads, sr, nr, p.state, p.coff, M, kp, 0);
  if (oop) {
    dim3 gg(wgs(M * pieces), (unsigned)L.rows);
    vq_evict_gather<<<gg, 256, 0, st>>>(rb, 0, rb, 0, pieces, wide ? 1 : 0, g, L.cap, L.cap, pcache, acc, pos, L.n_kv_heads,
                                        sr, M, kp, pcache_dst, acc_dst, pos_dst, L.cap, nullptr);
  } else {
    // through the staging area, 64 bytes of every row at a time (one pass, or two for 128-byte rows)
    NRes cnt;
    for (int b = 0; b < kMaxBatch; ++b) cnt.n[b] = M;
    for (int p0 = 0; p0 < pieces; p0 += 4) {
      const int wp = pieces - p0 < 4 ? pieces - p0 : 4;
      dim3 gg(wgs(M * wp), (unsigned)L.rows);
      vq_evict_gather<<<gg, 256, 0, st>>>(rb, p0, 64, 0, wp, wide ? 2 : 0, g, L.cap, L.cap, pcache, acc, pos, L.n_kv_heads, sr,
                                          M, kp, e.codes, e.acc, e.pos, M, p.state);
      vq_evict_copy_rows<<<gg, 256, 0, st>>>(64, 0, rb, p0, wp, wide ? 2 : 0, g, M, L.cap, L.n_kv_heads, sr, true, cnt,
                                             p.state, e.codes, e.acc, e.pos, M, pcache, acc, pos, L.cap);
    }
  }
  HCA_HIP(hipGetLastError());
  return HCA_OK;
}

// Sliced eviction for the step driver (out of place only): slice 0 prepares, every slice moves its
// share of the destination slots.
int32_t launch_evict_slice(const Layout& L, void* kcache, float* acc, int32_t* pos, const NRes& nr, int64_t nmax,
                           int64_t M, int64_t n_protect, void* ws, void* kcache_dst, float* acc_dst,
                           int32_t* pos_dst, int slice, int nslices, hipStream_t st) {
  // the plan is a pure function of the arguments, so it is rebuilt for every slice; only slice 0 launches
  // the preparation kernels
  EvictPlan pl;
  if (slice == 0) {
    int32_t rc = evict_prepare(L, kcache, acc, pos, nr, nmax, M, n_protect, nullptr, ws, kcache_dst, acc_dst, pos_dst, st, &pl);
    if (rc != HCA_OK) return rc;
  } else {
    SelRows& sr = pl.sr;
    pl.any = false;
    for (int b = 0; b < kMaxBatch; ++b) { sr.nsel[b] = 0; sr.want[b] = -1; }
    for (int b = 0; b < L.batch; ++b)
      if (nr.n[b] > M) { sr.nsel[b] = nr.n[b] - n_protect; sr.want[b] = M - n_protect; pl.any = true; }
    pl.oop = true;
    pl.M = M;
    carve(&pl.e, ws, L, M);
    pl.mblk = mblk_of(L, M);
    pl.kept = pl.e.kept;
    {
      SelectPlan p;
      select_plan(&p, pl.e.select, L.rows, nmax);
      pl.state = p.state;
    }
    pl.d.codes = (uint8_t*)kcache_dst;             pl.d.codes_row = L.codes_row_bytes();
    pl.d.meta = (uint8_t*)kcache_dst + L.meta_off;  pl.d.meta_row = L.meta_row_bytes();
    pl.d.acc = acc_dst; pl.d.pos = pos_dst; pl.d.ap_row = L.cap;
  }
  const int64_t per = (M + nslices - 1) / nslices;
  const int64_t d0 = per * slice;
  int64_t d1 = d0 + per;
  if (d1 > M) d1 = M;
  return evict_move(L, kcache, acc, pos, pl, d0, d1, st);
}

}  // namespace hca
