// Device-side building blocks shared by the HIP kernels of libhca: the tiled key-cache
// layout, the fixed-point query operand and the MFMA scoring of one 1 KiB code block.
// gfx950 only (wave64, v_mfma_i32_16x16x64_i8).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hca {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kHeadDim = 128;
constexpr int kBlockBytes = 1024;  // one code block = 64 lanes x 16 B
constexpr int kMetaBytes = 256;    // scales + zeros of one code block
constexpr int kMaxBatch = 64;

// Key cache in HBM.  A row (sequence, KV head) is a sequence of code blocks followed, in a
// second region, by the matching meta blocks.
//   4-bit / group 32: a block holds 16 tokens.  Lane l = t + 16*j (t token, j in 0..3) owns
//     bytes [16*l, 16*l+16): two 8-byte slots m = 0, 1; slot m packs channels
//     [32*(2m + j/2) + 16*(j%2), +16), two codes per byte, low nibble first.
//     Meta of token t: 16 B at 16*t = fp16 scale[0..3], zero[0..3].
//   2-bit / group 64: a block holds 32 tokens = two 16-token tiles u = 0, 1.  Lane l owns
//     bytes [16*l, +16): tile u at +8*u, slot m at +4*m; slot m packs channels
//     [64*m + 16*j, +16), four codes per byte, lowest bits first.
//     Meta of token (u, t): 8 B at 8*(16*u + t) = fp16 scale[0..1], zero[0..1].
// With this order one global_load_dwordx4 per lane fetches a whole block, fully coalesced,
// and every lane already holds the bytes it feeds to the matrix core.
struct Layout {
  int32_t bits, group, ng, tpb;  // ng groups per token, tpb tokens per block
  int32_t rows, gqa, batch, n_kv_heads;
  int64_t cap, nblk;             // capacity (tokens) and blocks per row
  int64_t meta_off;              // byte offset of the meta region
  __host__ __device__ int64_t codes_row_bytes() const { return nblk * kBlockBytes; }
  __host__ __device__ int64_t meta_row_bytes() const { return nblk * kMetaBytes; }
  __host__ __device__ int64_t total_bytes() const {
    return (int64_t)rows * (codes_row_bytes() + meta_row_bytes());
  }
};

struct NRes {  // resident tokens per sequence, passed by value to kernels
  int64_t n[kMaxBatch];
};

__device__ __forceinline__ float h2f(uint32_t bits16) {
  return (float)__builtin_bit_cast(_Float16, (unsigned short)(bits16 & 0xffffu));
}
__device__ __forceinline__ unsigned short f2h_bits(float x) {
  return __builtin_bit_cast(unsigned short, (_Float16)x);  // v_cvt_f16_f32, round to nearest even
}

// Codebook form: where the index of group `grp` sits in the stored record of slot `slot`, and back.
__device__ __forceinline__ int vq_byte_of(int grp, int64_t slot) {
  return (grp & ~15) | ((grp - (int)slot) & 15);
}
__device__ __forceinline__ int vq_group_at(int byte, int64_t slot) {
  return (byte & ~15) | ((byte + (int)slot) & 15);
}
// Wide codebook form: 16-bit indices, stored in tiles of kVqTile slots, group-major inside a tile
// (uint16 [row][tile][group][kVqTile]), so that the scan, which handles one group (or a few) at a time, reads
// each group's indices of its tile in one piece.  Position of (row, slot, group) in uint16 units:
constexpr int kVqTile = 16384;
__host__ __device__ __forceinline__ int64_t vq_tiles(int64_t cap) { return (cap + kVqTile - 1) / kVqTile; }
__host__ __device__ __forceinline__ int64_t vq_wide_at(int g, int64_t tiles, int64_t row, int64_t slot, int grp) {
  return ((row * tiles + slot / kVqTile) * g + grp) * kVqTile + slot % kVqTile;
}
// Power-of-two grid of one query head's table: s = 23 - floor(log2(largest magnitude)) (0 for an all-zero
// table), entry -> rint(entry * 2^s), at most 2^24 in magnitude, so that 64 of them add up exactly in 32 bits.
__device__ __forceinline__ int vq_grid_exponent(float amax) {
  return amax == 0.f ? 0 : 23 - ilogbf(amax);
}
__device__ __forceinline__ int vq_fix(float t, int s) { return (int)rintf(ldexpf(t, s)); }

// Order-preserving map float -> uint32 (larger float <=> larger key), -0 treated as +0.
__device__ __forceinline__ uint32_t order_key(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u << 1) == 0) u = 0;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// ---------------------------------------------------------------------------------------
// Query operand.  Each query head is mapped to fixed point, qfx = rint(q * 2^s) with
// s = 13 - floor(log2(max|q|)), split into a low and a high signed byte (qfx = lo + 256*hi).
// The A operand of the 16x16x64 i8 MFMA has 16 rows = 4 heads x 4 sub-rows; a sub-row is
// (byte piece, group selector) and carries the piece on the channels of its group and 0
// elsewhere, so one MFMA yields the per-group integer dot products of 16 tokens x 4 heads.
struct QShared {           // LDS image of the query of one row (4 heads)
  int16_t qfx[4][kHeadDim];
  int32_t qsum[4][4];      // per head, per group: sum of qfx
  int32_t sexp[4];
};

template <int BITS>
struct QOperand {
  v4i a[2];       // A operand of MFMA m = 0, 1
  float qf[4];    // (float) sum of qfx over group g, for head lane/16
  float unscale;  // 2^-s of head lane/16
  float nzero;    // -0.0f, opaque to the compiler (see zero_term)
};

// zero_g * Q_g rounded once, as a fused multiply-add with the addend -0.0f (x * y + (-0) == x * y for all finite
// x, y, signs of zero included): in this form the fp16 -> fp32 conversion of `zero` rides inside v_fma_mix_f32
// instead of costing an instruction of its own.  The addend is kept opaque so that it is not folded back.
__device__ __forceinline__ float zero_term(uint32_t zero_bits16, float qf, float nzero) {
  return __builtin_fmaf(h2f(zero_bits16), qf, nzero);
}

// channel held in byte x (0..15) of the B operand of MFMA m by a lane of k-group j
template <int BITS>
__device__ __forceinline__ int operand_channel(int m, int j, int x) {
  const int i = x >> 2, y = x & 3;
  if (BITS == 4) {
    const int idx = ((i >> 1) << 3) + 2 * y + (i & 1);
    return 32 * (2 * m + (j >> 1)) + 16 * (j & 1) + idx;
  } else {
    return 64 * m + 16 * j + 4 * y + i;
  }
}

// Computes the fixed-point query of row `row` into LDS.  Called by all threads of the block
// (at least 256); wave w < 4 handles query head w of the row.  Ends with a barrier.
__device__ __forceinline__ void load_query(const uint16_t* __restrict__ q, int row, int gqa, int group,
                                           QShared* sh) {
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  float x0 = 0.f, x1 = 0.f;
  if (w < gqa) {
    const uint32_t pr = reinterpret_cast<const uint32_t*>(q + ((int64_t)row * gqa + w) * kHeadDim)[lane];
    x0 = h2f(pr & 0xffffu);
    x1 = h2f(pr >> 16);
  }
  float amax = fmaxf(fabsf(x0), fabsf(x1));
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o));
  int s = 0;
  if (amax != 0.f) s = 13 - ilogbf(amax);
  if (w < 4) {                       // workgroups larger than four waves: the extra waves only take the barriers
    sh->qfx[w][2 * lane] = (int16_t)(int)rintf(ldexpf(x0, s));
    sh->qfx[w][2 * lane + 1] = (int16_t)(int)rintf(ldexpf(x1, s));
    if (lane == 0) sh->sexp[w] = s;
  }
  __syncthreads();
  if (tid < 16) {
    const int h = tid >> 2, g = tid & 3;
    int acc = 0;
    if (g * group < kHeadDim)
      for (int c = g * group; c < (g + 1) * group; ++c) acc += sh->qfx[h][c];
    sh->qsum[h][g] = acc;
  }
  __syncthreads();
}

template <int BITS>
__device__ __forceinline__ void build_operand(const QShared* sh, QOperand<BITS>* op) {
  const int lane = threadIdx.x & 63;
  const int r = lane & 15, j = lane >> 4;       // A operand: row r, k-group j
  const int head = r >> 2, sub = r & 3;
#pragma unroll
  for (int m = 0; m < 2; ++m) {
    int regs[4] = {0, 0, 0, 0};
    bool active;
    int piece;
    if (BITS == 4) { piece = sub & 1; active = ((sub >> 1) == (j >> 1)); }
    else           { piece = sub & 1; active = (sub < 2); }
    if (active) {
#pragma unroll
      for (int x = 0; x < 16; ++x) {
        const int v = sh->qfx[head][operand_channel<BITS>(m, j, x)];
        const int lo = ((v + 128) & 255) - 128;
        const int hi = (v - lo) / 256;
        const int b = (piece ? hi : lo) & 255;
        regs[x >> 2] |= b << (8 * (x & 3));
      }
    }
    op->a[m] = v4i{regs[0], regs[1], regs[2], regs[3]};
  }
  const int hd = lane >> 4;                      // epilogue: this lane scores head hd
#pragma unroll
  for (int g = 0; g < 4; ++g) op->qf[g] = (float)sh->qsum[hd][g];
  op->unscale = ldexpf(1.0f, -sh->sexp[hd]);
  float nz = -0.0f;
  asm volatile("" : "+v"(nz));
  op->nzero = nz;
}

// The same operand built once per workgroup of four waves instead of once per wave (every wave of a scan
// workgroup uses the same query): wave w forms two of the eight operand dwords of every lane, the image goes
// through LDS (img: 64 lanes x 8 dwords).  To be called by all 256 threads; contains a barrier.
template <int BITS>
__device__ __forceinline__ void build_operand_shared(const QShared* sh, uint32_t* img, QOperand<BITS>* op) {
  const int lane = threadIdx.x & 63, w = (threadIdx.x >> 6) & 3;
  const int r = lane & 15, j = lane >> 4;
  const int head = r >> 2, sub = r & 3;
  const int m = w >> 1;
  const int piece = sub & 1;
  const bool active = BITS == 4 ? ((sub >> 1) == (j >> 1)) : (sub < 2);
#pragma unroll
  for (int dd = 0; dd < 2; ++dd) {
    const int i = 2 * (w & 1) + dd;
    int reg = 0;
    if (active) {
#pragma unroll
      for (int y = 0; y < 4; ++y) {
        const int v = sh->qfx[head][operand_channel<BITS>(m, j, 4 * i + y)];
        const int lo = ((v + 128) & 255) - 128;
        const int hi = (v - lo) / 256;
        reg |= ((piece ? hi : lo) & 255) << (8 * y);
      }
    }
    img[lane * 8 + 4 * m + i] = (uint32_t)reg;
  }
  __syncthreads();
  const v4i* im = reinterpret_cast<const v4i*>(img + lane * 8);
  op->a[0] = im[0];
  op->a[1] = im[1];
  const int hd = lane >> 4;
#pragma unroll
  for (int g = 0; g < 4; ++g) op->qf[g] = (float)sh->qsum[hd][g];
  op->unscale = ldexpf(1.0f, -sh->sexp[hd]);
  float nz = -0.0f;
  asm volatile("" : "+v"(nz));
  op->nzero = nz;
}

__device__ __forceinline__ v4i mfma_i8(v4i a, v4i b, v4i c) {
  return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0);
}

// 4-bit: scores the 16 tokens of one block.  w = this lane's 16 code bytes, mw = the meta of
// token lane%16.  Returns z~ of (token lane%16, head lane/16).
__device__ __forceinline__ float score_block4(const QOperand<4>& op, uint4 w, uint4 mw) {
  const v4i zero = {0, 0, 0, 0};
  const uint32_t M = 0x0f0f0f0fu;
  v4i b0 = {(int)(w.x & M), (int)((w.x >> 4) & M), (int)(w.y & M), (int)((w.y >> 4) & M)};
  v4i b1 = {(int)(w.z & M), (int)((w.z >> 4) & M), (int)(w.w & M), (int)((w.w >> 4) & M)};
  v4i d0 = mfma_i8(op.a[0], b0, zero);   // rows: lo/hi of group 0, lo/hi of group 1
  v4i d1 = mfma_i8(op.a[1], b1, zero);   // rows: lo/hi of group 2, lo/hi of group 3
  const float t0 = fmaf(h2f(mw.x), (float)(d0.y * 256 + d0.x), zero_term(mw.z, op.qf[0], op.nzero));
  const float t1 = fmaf(h2f(mw.x >> 16), (float)(d0.w * 256 + d0.z), zero_term(mw.z >> 16, op.qf[1], op.nzero));
  const float t2 = fmaf(h2f(mw.y), (float)(d1.y * 256 + d1.x), zero_term(mw.w, op.qf[2], op.nzero));
  const float t3 = fmaf(h2f(mw.y >> 16), (float)(d1.w * 256 + d1.z), zero_term(mw.w >> 16, op.qf[3], op.nzero));
  const float a = t0 + t1, b = t2 + t3;
  return (a + b) * op.unscale;
}

// 2-bit: scores one 16-token tile.  c0, c1 = this lane's 4 code bytes of slot 0 and 1;
// mw = meta of the token (scale0|scale1<<16, zero0|zero1<<16).
__device__ __forceinline__ float score_tile2(const QOperand<2>& op, uint32_t c0, uint32_t c1, uint2 mw) {
  const v4i zero = {0, 0, 0, 0};
  const uint32_t M = 0x03030303u;
  v4i b0 = {(int)(c0 & M), (int)((c0 >> 2) & M), (int)((c0 >> 4) & M), (int)((c0 >> 6) & M)};
  v4i b1 = {(int)(c1 & M), (int)((c1 >> 2) & M), (int)((c1 >> 4) & M), (int)((c1 >> 6) & M)};
  v4i d0 = mfma_i8(op.a[0], b0, zero);   // rows: lo, hi of group 0
  v4i d1 = mfma_i8(op.a[1], b1, zero);   // rows: lo, hi of group 1
  const float t0 = fmaf(h2f(mw.x), (float)(d0.y * 256 + d0.x), zero_term(mw.y, op.qf[0], op.nzero));
  const float t1 = fmaf(h2f(mw.x >> 16), (float)(d1.y * 256 + d1.x), zero_term(mw.y >> 16, op.qf[1], op.nzero));
  return (t0 + t1) * op.unscale;
}

}  // namespace hca
