// Host-side declarations shared by the translation units of libhca.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <atomic>

#include "../../include/hca.h"

#include "hca_device.h"

namespace hca {

// Records a failing HIP status for hca_last_hip_error() and maps it to HCA_ERR_HIP.
int32_t hip_fail(hipError_t e);
#define HCA_HIP(call)                                  \
  do {                                                 \
    hipError_t e_ = (call);                            \
    if (e_ != hipSuccess) return ::hca::hip_fail(e_);  \
  } while (0)

// Validates `shape` and fills the layout; returns HCA_OK or an error code.
int32_t make_layout(const hca_shape* shape, Layout* L);
// Copies n_resident (host, [batch]) into `out` after range checks against the capacity.
int32_t load_nres(const Layout& L, const int64_t* n_resident, NRes* out, int64_t* nmax);

// Launch-shape knobs (defaults chosen by measurement on MI355X; hca_tune() overrides them).
struct Tuning {
  int gather_wgs = 0;      // workgroups of the value gather per row (0 = default)
  int gather_unroll = 4;   // rows in flight per thread
  int score_bpw = 0;       // 1 KiB code blocks per wave (0 = automatic; else kScoreBpwMin .. kScoreBpwMax)
  int score_depth = 0;     // blocks fetched ahead per wave (4 or 8; 0 = 8 for 4-bit codes, 4 for 2-bit)
  int host_spin_us = 100;  // how long the host-sum workers poll for the next call before they sleep
  int host_isa = 0;        // host_chunk_sum: 0 = the widest vector form the CPU has, 2 = the AVX2 form
  int select_wg = 0;       // threads per workgroup of the selection over the candidate lists: 1024 (pairs staged in
                           // LDS, needs a whole compute unit) or 256 (pairs read from L2, fits beside a running
                           // scan, but measured slower inside a decode step: its dependent passes crawl when a
                           // scan keeps the memory system busy); 0 = 1024
};
Tuning& tuning();
// Blocks per wave of the key scan.  The lower bound sizes the per-wave buffers of a launch (wall-clock stamps,
// partial softmax sums): a row of nblocks blocks never has more than nblocks / kScoreBpwMin + 4 waves.
constexpr int kScoreBpwMin = 4, kScoreBpwMax = 32;

inline int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// Raises a kernel's dynamic-LDS limit, once per device and call site (`done`: one bit per device).  Repeating
// the call on every launch is correct but stalls a host thread that is enqueueing ahead of the GPU.
inline int32_t lds_opt_in(const void* kernel, int bytes, std::atomic<uint64_t>* done) {
  int dev = 0;
  HCA_HIP(hipGetDevice(&dev));
  if (dev >= 0 && dev < 64 && ((done->load(std::memory_order_acquire) >> dev) & 1)) return HCA_OK;
  HCA_HIP(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
  if (dev >= 0 && dev < 64) done->fetch_or(1ull << dev, std::memory_order_release);
  return HCA_OK;
}

// Radix-select engine (select.hip): per row, finds the `want[r]`-th largest key among
// slots [0, nsel[r]) and per-chunk counts, so that a following ordered pass can emit the
// selected slots in ascending order.  See select.hip for the workspace carve-up.
struct SelectPlan {
  int64_t chunk;     // slots per chunk (one workgroup)
  int32_t nchunks;   // chunks per row (<= 1024)
  // workspace sub-buffers (device pointers)
  uint32_t* hist;    // [rows][3][2048]
  uint32_t* state;   // [rows][4]: key prefix, remaining count, (unused), (unused)
  uint32_t* ccount;  // [rows][nchunks][2]  (#greater, #equal) per chunk
  uint32_t* coff;    // [rows][nchunks][2]  exclusive prefix of ccount
};
struct SelRows {     // per-sequence selection parameters, by value
  int64_t nsel[kMaxBatch];   // slots [0, nsel) take part
  int64_t want[kMaxBatch];   // how many to select among them (0 < want <= nsel, or 0 = skip row)
};
size_t select_workspace_bytes(int rows, int64_t nmax);
size_t topk_workspace_bytes(int rows, int64_t cap);
void select_plan(SelectPlan* p, void* ws, int rows, int64_t nmax);
// Enqueues the selection passes over `vals` ([rows][stride] fp32).  Afterwards, for row r:
// state[r][0] = threshold key T, state[r][1] = number of slots with key == T to take (lowest first),
// coff = exclusive chunk prefixes of (#key > T, #key == T).
int32_t select_run(const SelectPlan& p, const float* vals, int64_t stride, int rows, int n_kv_heads,
                   const SelRows& sr, hipStream_t st);

int32_t launch_quantize(const Layout& L, void* kcache, const void* k_new, int64_t T, const NRes& nr,
                        float* acc_opt, int32_t* pos_opt, const NRes& vrow0, hipStream_t st);
int32_t launch_export(const Layout& L, const void* kcache, const NRes& nr, uint8_t* codes, void* scale,
                      void* zero, hipStream_t st);
int32_t launch_score(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax,
                     float* sel, float* z_opt, hipStream_t st, uint64_t* stamps = nullptr, const Tuning* tn = nullptr);
int64_t score_stamp_pairs(const Layout& L, int64_t nmax);
size_t score_workspace_bytes(const Layout& L);
int32_t launch_score_lse(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax,
                         float sm_scale, float* sel, float* lse_out, void* lse_ws, hipStream_t st);
int32_t launch_topk(const Layout& L, const float* sel, const NRes& nr, int64_t nmax, int32_t k,
                    int32_t* idx, int32_t* count, void* ws, hipStream_t st, bool hist_clean = false,
                    int64_t list_cap = 0);   // list_cap > 0: candidate lists carved for rows of that many slots
size_t topk_hist_bytes(int rows);
// Scan and selection in one: the scan keeps only the (order key, slot) pairs of the slots whose key reaches a
// per-row threshold estimated from a strided sample of the row, in per-chunk lists (chunk = the slots of one
// scan workgroup, at most kSelectMaxChunks of them per row).
constexpr int kSelectMaxChunks = 1024;
struct SelectOut {
  uint32_t* spec;       // [rows][4]: threshold key t0, 1 = the row has to be scanned again (with the threshold then
                        // in word 0), second threshold t1 <= t0 (only counted against), -
  uint32_t* ncand;      // [rows][kSelectMaxChunks] pairs in each chunk's list
  uint32_t* n1;         // [rows][kSelectMaxChunks] slots of each chunk with key >= t1
  uint2* lists;         // [rows][row_entries]: chunk c owns entries [c * chunk, (c + 1) * chunk)
  uint32_t* samples;    // [rows][m_samples] keys of the sampled slots (0: no such slot)
  int64_t row_entries;
  int m_samples;        // slots sampled per row (select_sample_count)
  uint32_t* mon;        // [rows][4] running figures of the selections on this workspace, or null (not kept)
};
constexpr int kSampleMax = 65536;
int select_sample_count(int64_t nmax, int32_t k);
// blocks per wave of the selecting scan over nmax slots (chunks per row <= kSelectMaxChunks); 0: too long a row
int select_scan_bpw(const Layout& L, int64_t nmax);
int32_t launch_select_sample(const Layout& L, const void* kcache, const void* q, const NRes& nr, int32_t k,
                             const SelectOut& so, hipStream_t st);
int32_t launch_select_scan(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax,
                           const SelectOut& so, bool only_failed, hipStream_t st, uint64_t* stamps = nullptr);
int32_t launch_select_sample_scores(const Layout& L, const void* kcache, const void* q, const NRes& nr,
                                    const SelectOut& so, hipStream_t st);
int32_t launch_select_rank_append(const Layout& L, void* kcache, const void* k_new, const NRes& nr_before, float* acc,
                                  int32_t* pos, const NRes& vrow0, int32_t k, const SelectOut& so, hipStream_t st);
// what a step's selecting scan of layer l carries for the layers behind it (null kcache: nothing)
struct SelectStepNext {
  void* a_kcache = nullptr;          // layer l + 1: threshold from its samples + append of its key
  const void* a_k_new = nullptr;
  float* a_acc = nullptr;
  int32_t* a_pos = nullptr;
  int64_t a_vrow0 = 0;
  int32_t k = 0;
  SelectOut a_so{};
  NRes a_nr{};                       // lengths before the layer's append
  const void* b_kcache = nullptr;    // layer l + 2: sampling
  const void* b_q = nullptr;
  SelectOut b_so{};
  NRes b_nr{};
};
int32_t launch_select_step(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax,
                           const SelectOut& so, hipStream_t st, uint64_t* stamps, const SelectStepNext& nx);
int32_t launch_select_step_pair(const Layout& L, const void* const kcache[2], const void* const q[2], const NRes nr[2],
                                const int64_t nmax[2], const SelectOut so[2], uint64_t* const stamps[2],
                                const SelectStepNext nx[2], hipStream_t st, hipEvent_t done = nullptr);
// the two layers of a pair launch, each with its selection workspace
int32_t launch_select_scan_step_pair(const Layout& L, const void* const kcache[2], const void* const q[2],
                                     const NRes nr[2], const int64_t nmax[2], int32_t k, void* const ws[2], hipStream_t st,
                                     uint64_t* const stamps[2], const SelectStepNext nx[2], hipEvent_t done = nullptr);
// the start of a step as two launches: sampling of up to four layers, threshold + append of up to two
int32_t launch_select_begin_samples(const Layout& L, int n, const void* const kcache[], const void* const q[],
                                    const NRes nr[], const SelectOut so[], hipStream_t st);
int32_t launch_select_begin_rank_append(const Layout& L, int n, void* const kcache[], const void* const k_new[],
                                        const NRes nr_before[], float* const acc[], int32_t* const pos[],
                                        int64_t vrow0, int32_t k, const SelectOut so[], hipStream_t st);
int32_t launch_select_rescan_pair(const Layout& L, const void* const kcache[2], const void* const q[2], const NRes nr[2],
                                  const int64_t nmax[2], const SelectOut so[2], hipStream_t st);
int32_t launch_select_finish_pair(const Layout& L, const void* const kcache[2], const void* const q[2], const NRes nr[2],
                                  const int64_t nmax[2], int32_t k, int32_t* const idx[2], int32_t* const count[2],
                                  void* const ws[2], hipStream_t st, bool small_wg = false);
// the SelectOut view of a selection workspace for rows of at most nmax_before slots (before the step's append)
SelectOut select_view(const Layout& L, void* ws, int64_t nmax_before, int32_t k);
int32_t launch_select_scan_step(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax,
                                int32_t k, void* ws, hipStream_t st, uint64_t* stamps, const SelectStepNext& nx);
int32_t launch_select_samples(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax,
                              int32_t k, void* ws, hipStream_t st);
int32_t launch_select_threshold_append(const Layout& L, void* kcache, const void* k_new, const NRes& nr_before,
                                       int64_t nmax_before, float* acc, int32_t* pos, const NRes& vrow0, int32_t k,
                                       void* ws, hipStream_t st);
int32_t launch_select_threshold(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax,
                                int32_t k, void* ws, hipStream_t st);
int32_t launch_select_begin(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax, int32_t k,
                            void* ws, hipStream_t st, uint64_t* stamps = nullptr);
int32_t launch_select_finish(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax, int32_t k,
                             int32_t* idx, int32_t* count, void* ws, hipStream_t st, bool small_wg = false);
int32_t launch_select_monitor(const Layout& L, void* ws, int32_t* out, int reset, hipStream_t st);
int32_t launch_select_report(const Layout& L, const NRes& nr, int64_t nmax, void* ws, int32_t* candidates,
                             int32_t* rescanned, hipStream_t st);
int32_t launch_score_topk(const Layout& L, const void* kcache, const void* q, const NRes& nr, int64_t nmax, int32_t k,
                          int32_t* idx, int32_t* count, void* ws, hipStream_t st);
int32_t launch_topp(const Layout& L, const float* sel, const NRes& nr, int64_t nmax, float sm_scale, double tau,
                    int32_t k_max, int32_t* idx, int32_t* count, uint64_t* mass_opt, void* ws, hipStream_t st);
size_t attend_workspace_bytes(const Layout& L, int64_t k);
int32_t launch_attend(const Layout& L, const void* kcache, const void* q, const int32_t* idx,
                      const int32_t* count, int32_t k, const int32_t* pos, const void* v_host,
                      int64_t host_stride, int64_t n_host_rows, const void* v_hbm, int64_t hbm_stride,
                      float sm_scale, float* y, float* acc_opt, void* ws, hipStream_t gst, hipStream_t st);
struct HostShare;
// first_entry: selected entries below it are left out (the host share of the value side sums them in place)
int32_t launch_gather(const Layout& L, const int32_t* idx, const int32_t* count, int32_t k, const int32_t* pos,
                      const void* v_host, int64_t host_stride, int64_t n_host_rows, const void* v_hbm,
                      int64_t hbm_stride, void* ws, hipStream_t st, uint64_t* stamps = nullptr, int first_entry = 0,
                      const Tuning* tn = nullptr,      // tn: launch-shape knobs (null: the process-wide ones)
                      const HostShare* hs = nullptr);  // hs: the launch also signals the host (hs->gpu_seq = hs->seq)
// (start, end) pairs a gather launch writes into `stamps` at most
constexpr int kGatherStampPairs = 1024;
constexpr int kAttendChunk = 256;   // selected tokens per chunk of the attend kernels
// Host share of the value side (Sec. 3.2 "CPU part", Eq. 5): the first `chunks` chunks of every row's selected
// tokens are summed on the host, where their value rows live; per token only exp(logit - chunk max) for each
// query head and the value-row number cross the link, and one partial sum per chunk and head comes back.
// All pointers are pinned host memory that the kernels read and write in place.
struct HostShare {
  int chunks = 0;                   // 0: off
  float* p = nullptr;               // [rows][chunks][4][kAttendChunk] weights relative to the chunk's maximum
  int32_t* vrow = nullptr;          // [rows][chunks][kAttendChunk] value row, -1: nothing to add for this entry
  const float* py = nullptr;        // [rows][chunks][4][kHeadDim] the host's partial sums
  const uint32_t* host_seq = nullptr;  // [rows]: the host stores `seq` here once the row's sums are in place
  uint32_t* gpu_seq = nullptr;      // [1]: `seq` once p / vrow are in place
  uint32_t* err = nullptr;          // [1]: set when a wait for the host ran out
  uint32_t seq = 0;
  int spin_limit = 0;               // polls of host_seq before the merge gives up
};

int host_share_chunks(int32_t k, int want);          // `want` clipped to the chunks k selected tokens make
size_t host_share_p_bytes(const Layout& L, int chunks);
size_t host_share_vrow_bytes(const Layout& L, int chunks);
size_t host_share_py_bytes(const Layout& L, int chunks);
// logits, chunk partials and the host's inputs of the first hs.chunks chunks of every row; the signal to the
// host comes from the next kernel on the stream (launch_gather with the same hs)
int32_t launch_attend_host_chunks(const Layout& L, const void* kcache, const void* q, const int32_t* idx,
                                  const int32_t* count, int32_t k, const int32_t* pos, int64_t n_host_rows,
                                  const void* v_hbm, int64_t hbm_stride, float sm_scale, void* ws, const HostShare& hs,
                                  hipStream_t st);
// host code (hostsum.hip): py[h][c] = sum over the chunk's entries with vrow >= 0 of p[h][i] * V[vrow[i]][c],
// h < G; entries with vrow >= n_rows are skipped and counted in the return value
int host_chunk_sum(int G, const float* p, const int32_t* vrow, const uint16_t* v_row0, int64_t n_rows, float* py);
int32_t launch_attend_gathered(const Layout& L, const void* kcache, const void* q, const int32_t* idx,
                               const int32_t* count, int32_t k, float sm_scale, float* y, float* acc_opt,
                               void* ws, hipStream_t st, const float* lse = nullptr, const HostShare* hs = nullptr);
int32_t launch_attend_weights(const Layout& L, const void* kcache, const void* q, const int32_t* idx,
                              const int32_t* count, int32_t k, const int32_t* pos, float sm_scale, const float* lse,
                              void* w_out, int32_t* vrow_out, float* acc_opt, void* ws, hipStream_t st);
int32_t launch_vq_attend_gathered(const Layout& L, int g, int c, const uint8_t* pcache, const float* lut,
                                  const int32_t* idx, const int32_t* count, int32_t k, float sm_scale, float* y,
                                  float* acc_opt, void* ws, hipStream_t st);
// codebook form of the key path (vq.hip).  Narrow: byte indices, table of a KV head in LDS (<= 128 KiB);
// wide: 16-bit indices, table read through L2.
inline bool vq_is_wide(const Layout& L, int g, int c) { return c > 256 || (int64_t)g * c * L.gqa > 32768; }
int32_t launch_vq_assign(const Layout& L, int g, int c, const float* centroids, uint8_t* pcache, const void* k_new,
                         int64_t T, const NRes& nr, float* acc_opt, int32_t* pos_opt, const NRes& vrow0, hipStream_t st);
int32_t launch_vq_score(const Layout& L, int g, int c, const float* centroids, const uint8_t* pcache, const void* q,
                        const NRes& nr, int64_t nmax, float* lut, float* sel, float* z_opt, hipStream_t st);
int32_t launch_vq_evict(const Layout& L, int g, int c, uint8_t* pcache, float* acc, int32_t* pos, const NRes& nr, int64_t nmax,
                        int64_t M, int64_t n_protect, int32_t* kept, void* ws, uint8_t* pcache_dst, float* acc_dst,
                        int32_t* pos_dst, hipStream_t st);
size_t evict_workspace_bytes(const Layout& L, int64_t M);
int32_t launch_evict(const Layout& L, void* kcache, float* acc, int32_t* pos, const NRes& nr,
                     int64_t nmax, int64_t M, int64_t n_protect, int32_t* kept, void* ws, void* kcache_dst,
                     float* acc_dst, int32_t* pos_dst, hipStream_t st);

int32_t launch_evict_slice(const Layout& L, void* kcache, float* acc, int32_t* pos, const NRes& nr, int64_t nmax,
                           int64_t M, int64_t n_protect, void* ws, void* kcache_dst, float* acc_dst,
                           int32_t* pos_dst, int slice, int nslices, hipStream_t st);

}  // namespace hca
