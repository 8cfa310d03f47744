// Host-side step driver: one decode step over all layers as a four-stage pipeline across layers
// (append + key scan | top-k | host-link gather | attend + eviction), one HIP stream per stage,
// stages of a layer chained by events.  Pure enqueue logic around the launchers of the other
// translation units; nothing here touches data.
#include <immintrin.h>

#include <atomic>
#include <chrono>
#include <condition_variable>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <mutex>
#include <thread>
#include <vector>

#include "hca_internal.h"

namespace hca {

// Host half of the hybrid value side (Sec. 3.2 "CPU part", Eq. 5): worker threads that, layer after layer, wait
// for the GPU's signal that a layer's weights and value-row numbers are in pinned memory, sum the host share's
// chunks from the value store where it lives, and store the step's sequence number per row for the GPU's merge
// to see.  Jobs are taken strictly in the order the step driver publishes them; every worker walks through
// every job (claiming whatever chunks are still unclaimed), so no queue is ever reordered.
class HostSide {
 public:
  static constexpr int kSlots = HCA_PIPELINE_MAX_PIPE, kRing = 1024;
  struct Job {
    uint32_t seq = 0;
    int slot = 0, chunks = 0;         // chunks per row of this job (<= the pipeline's host_chunks: k may be small)
    const uint16_t* v_host = nullptr;
    int64_t host_stride = 0, n_host_rows = 0;
    std::atomic<int> next_task{0};
    std::atomic<int> tasks_left{0};
    std::atomic<int64_t> t_first{0};  // when the first worker saw the GPU's signal (ns, steady clock)
    std::atomic<int> row_left[kMaxBatch * 8];
  };

  HostSide(const Layout& L, int chunks, int threads) : L_(L), chunks_(chunks), nthreads_(threads) {}
  ~HostSide() { stop(); release(); }

  // pinned control and exchange buffers (one set per pipeline slot), then the threads
  int32_t start() {
    if (L_.rows > kMaxBatch * 8) return HCA_ERR_UNSUPPORTED;
    const size_t pb = host_share_p_bytes(L_, chunks_), vb = host_share_vrow_bytes(L_, chunks_),
                 yb = host_share_py_bytes(L_, chunks_);
    for (int s = 0; s < kSlots; ++s) {
      HCA_HIP(hipHostMalloc((void**)&p_[s], pb, hipHostMallocCoherent));
      HCA_HIP(hipHostMalloc((void**)&vrow_[s], vb, hipHostMallocCoherent));
      HCA_HIP(hipHostMalloc((void**)&py_[s], yb, hipHostMallocCoherent));
      std::memset(py_[s], 0, yb);
    }
    // flags: one cache line each, so that the GPU's store to one never touches a line the host is writing
    HCA_HIP(hipHostMalloc((void**)&flags_, kFlagBytes, hipHostMallocCoherent));
    std::memset(flags_, 0, kFlagBytes);
    jobs_.reset(new Job[kRing]);
    progress_.reset(new std::atomic<uint32_t>[nthreads_ > 0 ? nthreads_ : 1]);
    for (int t = 0; t < nthreads_; ++t) progress_[t].store(1, std::memory_order_relaxed);
    for (int t = 0; t < nthreads_; ++t) threads_.emplace_back([this, t] { loop(t); });
    return HCA_OK;
  }

  // What the kernels of the job with number `seq` in slot `slot` get
  HostShare share(int slot, uint32_t seq, int spin_limit) const {
    HostShare h;
    h.chunks = chunks_;
    h.p = p_[slot];
    h.vrow = vrow_[slot];
    h.py = py_[slot];
    h.host_seq = host_seq(slot);
    h.gpu_seq = gpu_seq(slot);
    h.err = err_word();
    h.seq = seq;
    h.spin_limit = spin_limit;
    return h;
  }

  uint32_t next_seq() const { return published_.load(std::memory_order_relaxed) + 1; }

  // Called by the enqueueing thread after the layer's host-chunk kernels are enqueued.
  void publish(uint32_t seq, int slot, int chunks, const void* v_host, int64_t host_stride, int64_t n_host_rows) {
    // the ring entry is free once every worker has gone past the job that used it last
    if (seq > (uint32_t)kRing) {
      const uint32_t old = seq - kRing;
      for (int t = 0; t < nthreads_; ++t)
        while ((int32_t)(progress_[t].load(std::memory_order_acquire) - old) <= 0) _mm_pause();
    }
    Job& j = jobs_[seq % kRing];
    j.seq = seq;
    j.slot = slot;
    j.chunks = chunks;
    j.v_host = (const uint16_t*)v_host;
    j.host_stride = host_stride;
    j.n_host_rows = n_host_rows;
    j.next_task.store(0, std::memory_order_relaxed);
    j.tasks_left.store(L_.rows * chunks, std::memory_order_relaxed);
    j.t_first.store(0, std::memory_order_relaxed);
    for (int r = 0; r < L_.rows; ++r) j.row_left[r].store(chunks, std::memory_order_relaxed);
    published_.store(seq, std::memory_order_release);
    if (sleepers_.load(std::memory_order_acquire) > 0) {
      std::lock_guard<std::mutex> g(m_);
      cv_.notify_all();
    }
  }

  uint32_t errors() const { return __atomic_load_n(err_word(), __ATOMIC_RELAXED) != 0 ? 1u : 0u; }
  uint32_t bad_rows() const { return bad_rows_.load(std::memory_order_relaxed); }
  // mean time from the GPU's signal (as first seen by a worker) to the job's last chunk, and mean time per chunk
  void times(double* job_us, double* task_us) const {
    const int64_t nj = jobs_done_.load(std::memory_order_relaxed), nt = tasks_done_.load(std::memory_order_relaxed);
    *job_us = nj > 0 ? job_ns_.load(std::memory_order_relaxed) * 1e-3 / (double)nj : 0.0;
    *task_us = nt > 0 ? task_ns_.load(std::memory_order_relaxed) * 1e-3 / (double)nt : 0.0;
  }

  void stop() {
    if (stopped_) return;
    stopped_ = true;
    stop_.store(true, std::memory_order_release);
    {
      std::lock_guard<std::mutex> g(m_);
      cv_.notify_all();
    }
    for (auto& t : threads_) t.join();
    threads_.clear();
  }

 private:
  static constexpr size_t kLine = 64;
  // flags_: [kSlots] gpu_seq lines, then [kSlots][rows] host_seq (a line per slot and 16 rows), then the error word
  static constexpr size_t kFlagBytes = kLine * (kSlots + kSlots * (kMaxBatch * 8 / 16) + 1);
  uint32_t* gpu_seq(int slot) const { return (uint32_t*)(flags_ + kLine * slot); }
  uint32_t* host_seq(int slot) const { return (uint32_t*)(flags_ + kLine * (kSlots + slot * (kMaxBatch * 8 / 16))); }
  uint32_t* err_word() const { return (uint32_t*)(flags_ + kLine * (kSlots + kSlots * (kMaxBatch * 8 / 16))); }

  void release() {
    for (int s = 0; s < kSlots; ++s) {
      if (p_[s]) (void)hipHostFree(p_[s]);
      if (vrow_[s]) (void)hipHostFree(vrow_[s]);
      if (py_[s]) (void)hipHostFree(py_[s]);
      p_[s] = nullptr; vrow_[s] = nullptr; py_[s] = nullptr;
    }
    if (flags_) (void)hipHostFree(flags_);
    flags_ = nullptr;
  }

  void loop(int me) {
    // Weights far below the chunk's maximum are subnormal floats; x86 cores take a microcode assist for every
    // operation on one (a hundred times the cost of a normal multiply-add).  Flush them to zero in this thread:
    // what is lost is below 2^-126 of the chunk's largest weight.
    _mm_setcsr(_mm_getcsr() | 0x8040u);               // FTZ | DAZ
    uint32_t next = 1;
    for (;;) {
      // 1. the job's description
      int idle = 0;
      while ((int32_t)(published_.load(std::memory_order_acquire) - next) < 0) {
        if (stop_.load(std::memory_order_acquire)) return;
        if (++idle < 20000) { _mm_pause(); continue; }
        std::unique_lock<std::mutex> g(m_);               // nothing for a while: sleep until the next publish
        sleepers_.fetch_add(1, std::memory_order_acq_rel);
        cv_.wait_for(g, std::chrono::milliseconds(50), [&] {
          return stop_.load(std::memory_order_acquire) ||
                 (int32_t)(published_.load(std::memory_order_acquire) - next) >= 0;
        });
        sleepers_.fetch_sub(1, std::memory_order_acq_rel);
        idle = 0;
      }
      Job& j = jobs_[next % kRing];
      // 2. the GPU's signal that the job's inputs are in pinned memory
      const uint32_t* gs = gpu_seq(j.slot);
      while ((int32_t)(__atomic_load_n(gs, __ATOMIC_ACQUIRE) - j.seq) < 0) {
        if (stop_.load(std::memory_order_acquire)) return;
        _mm_pause();
      }
      // 3. chunks, one at a time, whoever comes first
      const int nch = j.chunks, ntask = L_.rows * nch;
      int64_t t_seen = now_ns(), zero = 0;
      j.t_first.compare_exchange_strong(zero, t_seen, std::memory_order_acq_rel);
      for (int t = j.next_task.fetch_add(1, std::memory_order_acq_rel); t < ntask;
           t = j.next_task.fetch_add(1, std::memory_order_acq_rel)) {
        const int64_t t_a = now_ns();
        const int row = t / nch, ch = t % nch;
        const int64_t e = (int64_t)row * nch + ch;
        const int bad = host_chunk_sum(L_.gqa, p_[j.slot] + e * 4 * kAttendChunk, vrow_[j.slot] + e * kAttendChunk,
                                       j.v_host + (int64_t)row * j.host_stride * kHeadDim,
                                       j.n_host_rows < j.host_stride ? j.n_host_rows : j.host_stride,
                                       py_[j.slot] + e * 4 * kHeadDim);
        if (bad) bad_rows_.fetch_add((uint32_t)bad, std::memory_order_relaxed);
        if (j.row_left[row].fetch_sub(1, std::memory_order_acq_rel) == 1)      // the row's last chunk: tell the GPU
          __atomic_store_n(host_seq(j.slot) + row, j.seq, __ATOMIC_RELEASE);
        const int64_t t_b = now_ns();
        task_ns_.fetch_add(t_b - t_a, std::memory_order_relaxed);
        tasks_done_.fetch_add(1, std::memory_order_relaxed);
        if (j.tasks_left.fetch_sub(1, std::memory_order_acq_rel) == 1) {
          job_ns_.fetch_add(t_b - j.t_first.load(std::memory_order_acquire), std::memory_order_relaxed);
          jobs_done_.fetch_add(1, std::memory_order_relaxed);
        }
      }
      ++next;
      progress_[me].store(next, std::memory_order_release);
    }
  }

  static int64_t now_ns() {
    return std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now().time_since_epoch()).count();
  }
  std::atomic<int64_t> job_ns_{0}, task_ns_{0}, jobs_done_{0}, tasks_done_{0};
  Layout L_;
  int chunks_, nthreads_;
  float* p_[kSlots] = {};
  int32_t* vrow_[kSlots] = {};
  float* py_[kSlots] = {};
  unsigned char* flags_ = nullptr;
  std::unique_ptr<Job[]> jobs_;
  std::unique_ptr<std::atomic<uint32_t>[]> progress_;
  std::atomic<uint32_t> published_{0};
  std::atomic<uint32_t> bad_rows_{0};
  std::atomic<int> sleepers_{0};
  std::atomic<bool> stop_{false};
  bool stopped_ = false;
  std::mutex m_;
  std::condition_variable cv_;
  std::vector<std::thread> threads_;
};

}  // namespace hca

struct hca_pipeline {
  hca::Layout L;
  int n_layers;
  hca_pipeline_desc d;
  int n_sel;                        // score buffers in use (<= n_layers)
  bool sel_waits;                   // fewer score buffers than layers: the scan waits for the buffer's last top-k
  std::vector<hipEvent_t> score_done, sel_free;
  int timing_stride;
  hipEvent_t topk_done[HCA_PIPELINE_MAX_PIPE], gather_done[HCA_PIPELINE_MAX_PIPE], pipe_free[HCA_PIPELINE_MAX_PIPE];
  int n_pipe;                       // sets of selection / staging buffers in use
  hipEvent_t slot_free[HCA_PIPELINE_MAX_PIPE];   // what frees each set: the layer_done of the layer that used it last,
                                    // or the set's pipe_free when that layer's layer_done comes later (sliced
                                    // eviction); null: never used
  bool dual;                        // fused selection on two streams: even layers on stream_scan, odd on stream_topk
  bool pair;                        // fused selection, one scan launch per two layers
  std::vector<hipEvent_t> layer_done;
  std::vector<hipEvent_t> t0, t1;   // timing events around the scan launches: [slots][layers]
  int timing_slots;
  std::unique_ptr<hca::HostSide> host;   // hybrid value side (desc.host_chunks > 0), else null
  int host_chunks = 0, host_spin_limit = 0;
  hca::Tuning tune;                 // this pipeline's launch-shape knobs
};

// an eviction in progress: its slices go out one at a time behind the attends of the following layers
struct EvictJob {
  bool active = false;
  int layer = 0, next_slice = 0;
  hca::NRes nr;
  int64_t nmax = 0, M = 0;
};
constexpr int kEvictSlices = 6;

using namespace hca;

extern "C" {

hca_pipeline* hca_pipeline_create(const hca_shape* shape, int32_t n_layers, const hca_pipeline_desc* desc,
                                  int32_t timing_slots) {
  Layout L;
  if (make_layout(shape, &L) != HCA_OK || desc == nullptr || n_layers < 1 || timing_slots < 0) return nullptr;
  if (desc->n_sel < 3 || desc->n_sel > HCA_PIPELINE_MAX_SEL) return nullptr;
  const bool fused = desc->fused_select != 0;
  for (int i = 0; i < desc->n_sel; ++i) if ((fused ? desc->ws_select[i] : (void*)desc->sel[i]) == nullptr) return nullptr;
  if (fused && (desc->vq_groups != 0 || desc->topp_tau > 0.0)) return nullptr;   // uniform codes and top-k only
  // two scan streams: only with the fused selection, and with enough selection workspaces that the three layers a
  // launch touches on either stream never share one
  if (desc->dual_scan < 0 || desc->dual_scan > 2) return nullptr;
  if (desc->dual_scan != 0 && (!fused || (desc->n_sel < 6 && desc->n_sel < n_layers))) return nullptr;
  const int n_pipe = desc->n_pipe == 0 ? 4 : desc->n_pipe;
  if (n_pipe < 4 || n_pipe > HCA_PIPELINE_MAX_PIPE) return nullptr;
  const bool own_idx = desc->layer_idx != nullptr;
  if (own_idx && (desc->layer_count == nullptr || desc->layer_idx_stride < 1)) return nullptr;
  for (int i = 0; i < n_pipe; ++i)
    if ((!own_idx && (desc->idx[i] == nullptr || desc->count[i] == nullptr)) || desc->ws_attend[i] == nullptr) return nullptr;
  if (desc->ws_topk == nullptr) return nullptr;
  if (desc->vq_groups != 0) {                // codebook form: same limits as the hca_vq_* calls; eviction in place
    if (desc->vq_groups != 32 && desc->vq_groups != 64) return nullptr;
    if (desc->vq_codewords < 1 || desc->vq_codewords > 8192) return nullptr;
    if (desc->spare_kcache != nullptr || desc->spare_acc != nullptr || desc->spare_pos != nullptr) return nullptr;
  }
  if (!(desc->topp_tau >= 0.0)) return nullptr;
  if (desc->host_chunks < 0 || desc->host_chunks > 64 || desc->host_threads < 0 || desc->host_threads > 64 ||
      desc->host_spin_limit < 0)
    return nullptr;
  if (desc->host_chunks > 0 && desc->vq_groups != 0) return nullptr;          // uniform codes only
  if (desc->gather_wgs < 0 || desc->gather_wgs > 1024 || desc->gather_unroll < 0 || desc->gather_unroll > 4) return nullptr;
  if (desc->score_bpw != 0 && (desc->score_bpw < kScoreBpwMin || desc->score_bpw > kScoreBpwMax)) return nullptr;
  if (!(desc->score_depth == 0 || desc->score_depth == 4 || desc->score_depth == 8)) return nullptr;
  if (!(desc->select_wg == 0 || desc->select_wg == 256 || desc->select_wg == 1024)) return nullptr;
  hca_pipeline* p = new hca_pipeline();
  p->L = L;
  p->n_layers = n_layers;
  p->d = *desc;
  p->timing_slots = timing_slots;
  p->n_pipe = n_pipe;
  for (int i = 0; i < HCA_PIPELINE_MAX_PIPE; ++i) p->slot_free[i] = nullptr;
  p->dual = desc->dual_scan == 1;
  p->pair = desc->dual_scan == 2;
  p->n_sel = desc->n_sel < n_layers ? desc->n_sel : n_layers;
  p->sel_waits = desc->n_sel < n_layers;
  p->timing_stride = desc->timing_layer_stride > 1 ? desc->timing_layer_stride : 1;
  p->tune = tuning();                        // the process-wide defaults, then this pipeline's own values
  if (desc->gather_wgs > 0) p->tune.gather_wgs = desc->gather_wgs;
  if (desc->gather_unroll > 0) p->tune.gather_unroll = desc->gather_unroll;
  if (desc->score_bpw > 0) p->tune.score_bpw = desc->score_bpw;
  if (desc->score_depth > 0) p->tune.score_depth = desc->score_depth;
  if (desc->select_wg > 0) p->tune.select_wg = desc->select_wg;
  p->host_chunks = desc->host_chunks;
  // ~2 us per poll over the host link: about a second before a merge gives up on the host
  p->host_spin_limit = desc->host_spin_limit > 0 ? desc->host_spin_limit : (1 << 19);
  p->score_done.resize(p->n_sel);
  p->sel_free.resize(p->n_sel);
  bool ok = true;
  auto mk = [&](hipEvent_t* e, unsigned flags) { ok = ok && hipEventCreateWithFlags(e, flags) == hipSuccess; };
  for (int i = 0; i < p->n_sel; ++i) { mk(&p->score_done[i], hipEventDisableTiming); mk(&p->sel_free[i], hipEventDisableTiming); }
  for (int i = 0; i < HCA_PIPELINE_MAX_PIPE; ++i) {
    mk(&p->topk_done[i], hipEventDisableTiming);
    mk(&p->gather_done[i], hipEventDisableTiming);
    mk(&p->pipe_free[i], hipEventDisableTiming);
  }
  p->layer_done.resize(n_layers);
  for (int l = 0; l < n_layers; ++l) mk(&p->layer_done[l], hipEventDisableTiming);
  p->t0.resize((size_t)timing_slots * n_layers);
  p->t1.resize((size_t)timing_slots * n_layers);
  for (size_t i = 0; i < p->t0.size(); ++i) { mk(&p->t0[i], hipEventDefault); mk(&p->t1[i], hipEventDefault); }
  if (!ok) { delete p; return nullptr; }   // events already made are left to process teardown
  if (p->host_chunks > 0) {
    p->host.reset(new HostSide(L, p->host_chunks, desc->host_threads));
    if (p->host->start() != HCA_OK) { delete p; return nullptr; }
  }
  // the top-k histogram at the head of ws_topk starts clean and is kept clean by every selection
  if (hipMemsetAsync(desc->ws_topk, 0, topk_hist_bytes(L.rows), (hipStream_t)desc->stream_topk) != hipSuccess) {
    delete p;
    return nullptr;
  }
  return p;
}

void hca_pipeline_destroy(hca_pipeline* p) {
  if (p == nullptr) return;
  if (p->host) {                       // the workers read pinned buffers that die with the object
    (void)hipDeviceSynchronize();      // no merge may still be polling a flag of theirs
    p->host->stop();
  }
  for (auto e : p->score_done) (void)hipEventDestroy(e);
  for (auto e : p->sel_free) (void)hipEventDestroy(e);
  for (int i = 0; i < HCA_PIPELINE_MAX_PIPE; ++i) {
    (void)hipEventDestroy(p->topk_done[i]);
    (void)hipEventDestroy(p->gather_done[i]);
    (void)hipEventDestroy(p->pipe_free[i]);
  }
  for (auto e : p->layer_done) (void)hipEventDestroy(e);
  for (auto e : p->t0) (void)hipEventDestroy(e);
  for (auto e : p->t1) (void)hipEventDestroy(e);
  delete p;
}

int32_t hca_pipeline_step(hca_pipeline* p, hca_layer* layers, int64_t* n_resident, int64_t value_row0, int32_t k,
                          int64_t host_stride, int64_t n_host_rows, int64_t hbm_stride, float sm_scale,
                          const int64_t* evict_M, int64_t n_protect, int32_t timing_slot) {
  if (p == nullptr || layers == nullptr || n_resident == nullptr) return HCA_ERR_BAD_ARG;
  const Layout& L = p->L;
  if (k < 1 || k > L.cap || k > 64 * 256) return HCA_ERR_CAPACITY;
  if (p->d.layer_idx != nullptr && p->d.layer_idx_stride < (int64_t)L.rows * k) return HCA_ERR_CAPACITY;
  for (int l = 0; evict_M != nullptr && l < p->n_layers; ++l) {
    if (evict_M[l] == 0) continue;
    if (evict_M[l] < 1 || evict_M[l] > L.cap || n_protect < 0 || n_protect > evict_M[l]) return HCA_ERR_CAPACITY;
    if (p->d.ws_evict == nullptr) return HCA_ERR_BAD_ARG;
    const int spare = (p->d.spare_kcache != nullptr) + (p->d.spare_acc != nullptr) + (p->d.spare_pos != nullptr);
    if (spare != 0 && spare != 3) return HCA_ERR_BAD_ARG;
  }
  if (timing_slot >= p->timing_slots) return HCA_ERR_BAD_ARG;
  const int vg = p->d.vq_groups, vc = p->d.vq_codewords;
  const bool vq = vg > 0;
  // Every argument, length and capacity check of every layer comes before the first enqueue, so that an error
  // found here leaves the streams, n_resident and layers[] untouched.  Past this loop only a failing HIP call can
  // end the step early.
  if (n_host_rows < 0 || host_stride < 0 || hbm_stride < 0) return HCA_ERR_BAD_ARG;
  for (int l = 0; l < p->n_layers; ++l) {
    const hca_layer& ly = layers[l];
    if (ly.kcache == nullptr || ly.acc == nullptr || ly.pos == nullptr || ly.k_new == nullptr || ly.q == nullptr ||
        ly.y == nullptr)
      return HCA_ERR_BAD_ARG;
    if (vq && (ly.vq_centroids == nullptr || ly.vq_lut == nullptr)) return HCA_ERR_BAD_ARG;
    if (n_host_rows > 0 && (ly.v_host == nullptr || host_stride < n_host_rows)) return HCA_ERR_BAD_ARG;
    if (ly.v_host == nullptr && ly.v_hbm == nullptr) return HCA_ERR_BAD_ARG;
    NRes nr;
    int64_t nmax;
    const int32_t rc = load_nres(L, n_resident + (int64_t)l * L.batch, &nr, &nmax);
    if (rc != HCA_OK) return rc;
    for (int b = 0; b < L.batch; ++b)
      if (nr.n[b] + 1 > L.cap) return HCA_ERR_CAPACITY;             // the step appends one token per sequence
    if (!vq && timing_slot >= 0 && p->d.scan_stamps != nullptr && p->d.scan_stamp_pairs < score_stamp_pairs(L, nmax + 1))
      return HCA_ERR_CAPACITY;
    if (p->d.fused_select != 0 && select_scan_bpw(L, nmax + 1) == 0) return HCA_ERR_CAPACITY;   // row too long for the lists
    if (p->host_chunks > 0 && (ly.v_host == nullptr || n_host_rows < 1)) return HCA_ERR_BAD_ARG;  // the host sums from v_host
  }
  const int hchunks = p->host ? host_share_chunks(k, p->host_chunks) : 0;
  const hipStream_t sa = (hipStream_t)p->d.stream_scan, sb = (hipStream_t)p->d.stream_topk, sb_topk = sb;
  hipStream_t sg = (hipStream_t)p->d.stream_gather, sc = (hipStream_t)p->d.stream_attend;
  NRes vrow0;
  for (int b = 0; b < kMaxBatch; ++b) vrow0.n[b] = value_row0;
  EvictJob job;
  // enqueues the next slice of `j` on the attend stream; the last slice swaps the layer's buffers with
  // the spare set and releases the layer for the next step
  auto advance = [&](EvictJob& j) -> int32_t {
    hca_layer& jl = layers[j.layer];
    int32_t rc = launch_evict_slice(L, jl.kcache, jl.acc, jl.pos, j.nr, j.nmax, j.M, n_protect, p->d.ws_evict,
                                    p->d.spare_kcache, p->d.spare_acc, p->d.spare_pos, j.next_slice, kEvictSlices, sc);
    if (rc != HCA_OK) return rc;
    if (++j.next_slice == kEvictSlices) {
      void* ok = jl.kcache; float* oa = jl.acc; int32_t* op = jl.pos;
      jl.kcache = p->d.spare_kcache; jl.acc = p->d.spare_acc; jl.pos = p->d.spare_pos;
      p->d.spare_kcache = ok; p->d.spare_acc = oa; p->d.spare_pos = op;
      HCA_HIP(hipEventRecord(p->layer_done[j.layer], sc));
      j.active = false;
    }
    return HCA_OK;
  };
  const bool fused = p->d.fused_select != 0;
  // Fused selection: the scan stream carries one launch per layer.  The launch of layer l is its selecting scan
  // plus a few workgroups for the layers behind it: the threshold of layer l + 1 (from samples the previous launch
  // took) with the append of its key, and the sampling of layer l + 2.  The first two layers' samples and the first
  // layer's threshold + append come from launches of their own at the start of the step.
  auto lengths = [&](int l2, NRes* out, int64_t* nmax2) -> int32_t {
    const hca_layer& y2 = layers[l2];
    if (y2.kcache == nullptr || y2.acc == nullptr || y2.pos == nullptr || y2.k_new == nullptr || y2.q == nullptr)
      return HCA_ERR_BAD_ARG;
    const int32_t rc = load_nres(L, n_resident + (int64_t)l2 * L.batch, out, nmax2);
    if (rc != HCA_OK) return rc;
    for (int b = 0; b < L.batch; ++b)
      if (out->n[b] + 1 > L.cap) return HCA_ERR_CAPACITY;
    return HCA_OK;
  };
  // before anything of this step touches layer l2's cache or its selection workspace
  // Two scan streams (desc.dual_scan): even layers run append + scan + selection on stream_scan, odd layers on
  // stream_topk, each stream a chain of its own (a launch carries the threshold + append of the layer two on and
  // the sampling of the layer four on), so that one stream's scan fills the time the other spends between two
  // of its scans (launch gap, selection) and the key stream from HBM does not pause.
  // Paired launches (desc.dual_scan == 2): the same two chains, but layers l and l + 1 (l even) share one launch
  // on stream_scan, and their selections follow each other on stream_topk.
  const int S = (p->dual || p->pair) ? 2 : 1;
  auto scan_stream = [&](int l2) -> hipStream_t { return (p->dual && (l2 & 1)) ? sb : sa; };
  auto wait_layer = [&](int l2) -> int32_t {
    if (p->sel_waits) HCA_HIP(hipStreamWaitEvent(scan_stream(l2), p->sel_free[l2 % p->n_sel], 0));
    HCA_HIP(hipStreamWaitEvent(scan_stream(l2), p->layer_done[l2], 0));
    return HCA_OK;
  };
  bool begun = false;                      // the chains' first layers already have their threshold + append
  if (fused && !p->dual) {
    // one stream carries every chain: the step starts with two launches, the sampling of the first layers of
    // every chain and the threshold + append of the chains' first layers
    const int ns = 2 * S < p->n_layers ? 2 * S : p->n_layers, nt = S < p->n_layers ? S : p->n_layers;
    const void* kc[4];
    const void* qq[4];
    NRes nrs[4];
    SelectOut sos[4];
    // layer_done events are recorded in layer order on the attend stream (not so with spare-buffer evictions, whose
    // last slice records it later): the wait for the last of these layers then covers the others
    const bool one_wait = !p->sel_waits && p->d.spare_kcache == nullptr;
    for (int l2 = 0; l2 < ns; ++l2) {
      int64_t m2;
      int32_t rc = lengths(l2, &nrs[l2], &m2);
      if (rc != HCA_OK) return rc;
      if (!one_wait || l2 == ns - 1) rc = wait_layer(l2);
      if (rc != HCA_OK) return rc;
      kc[l2] = layers[l2].kcache;
      qq[l2] = layers[l2].q;
      sos[l2] = select_view(L, p->d.ws_select[l2 % p->n_sel], m2, k);
    }
    int32_t rc = launch_select_begin_samples(L, ns, kc, qq, nrs, sos, sa);
    if (rc != HCA_OK) return rc;
    void* kcw[2];
    const void* kn[2];
    float* accs[2];
    int32_t* poss[2];
    for (int l2 = 0; l2 < nt; ++l2) {
      kcw[l2] = layers[l2].kcache;
      kn[l2] = layers[l2].k_new;
      accs[l2] = layers[l2].acc;
      poss[l2] = layers[l2].pos;
    }
    rc = launch_select_begin_rank_append(L, nt, kcw, kn, nrs, accs, poss, value_row0, k, sos, sa);
    if (rc != HCA_OK) return rc;
    begun = true;
  } else if (fused) {
    for (int l2 = 0; l2 < 2 * S && l2 < p->n_layers; ++l2) {
      NRes n2;
      int64_t m2;
      int32_t rc = lengths(l2, &n2, &m2);
      if (rc != HCA_OK) return rc;
      rc = wait_layer(l2);
      if (rc != HCA_OK) return rc;
      rc = launch_select_samples(L, layers[l2].kcache, layers[l2].q, n2, m2, k, p->d.ws_select[l2 % p->n_sel],
                                 scan_stream(l2));
      if (rc != HCA_OK) return rc;
    }
  }
  // What the fused scan launch of a layer needs: its lengths after the append, its stamp area, and the jobs it
  // carries for the layers behind it on its chain.  Enqueues what has to precede the launch (the first layers'
  // own threshold + append, the waits for the layer whose sampling rides along) and moves the host's lengths on.
  struct FusedCtx { NRes nr; int64_t nmax = 0; uint64_t* stamps = nullptr; SelectStepNext nx; };
  auto fused_prepare = [&](int l, FusedCtx* c) -> int32_t {
    hca_layer& ly = layers[l];
    int64_t* nl = n_resident + (int64_t)l * L.batch;
    const hipStream_t st = scan_stream(l);
    int32_t rc = load_nres(L, nl, &c->nr, &c->nmax);
    if (rc != HCA_OK) return rc;
    // (the waits for this layer's buffers went out before its sampling; its threshold and append rode on an
    // earlier launch of its chain, except for the chain's first layer)
    if (l < S && !begun) {
      rc = launch_select_threshold_append(L, ly.kcache, ly.k_new, c->nr, c->nmax, ly.acc, ly.pos, vrow0, k,
                                          p->d.ws_select[l % p->n_sel], st);
      if (rc != HCA_OK) return rc;
    }
    for (int b = 0; b < L.batch; ++b) { c->nr.n[b] += 1; nl[b] += 1; }
    c->nmax += 1;
    if (timing_slot >= 0 && p->d.scan_stamps != nullptr)
      c->stamps = (uint64_t*)p->d.scan_stamps + ((int64_t)timing_slot * p->n_layers + l) * p->d.scan_stamp_pairs * 2;
    SelectStepNext& nx = c->nx;
    nx.k = k;
    if (l + S < p->n_layers) {
      hca_layer& ya = layers[l + S];
      int64_t ma;
      rc = lengths(l + S, &nx.a_nr, &ma);
      if (rc != HCA_OK) return rc;
      nx.a_kcache = ya.kcache;
      nx.a_k_new = ya.k_new;
      nx.a_acc = ya.acc;
      nx.a_pos = ya.pos;
      nx.a_vrow0 = value_row0;
      nx.a_so = select_view(L, p->d.ws_select[(l + S) % p->n_sel], ma, k);
    }
    if (l + 2 * S < p->n_layers) {
      int64_t mb;
      rc = lengths(l + 2 * S, &nx.b_nr, &mb);
      if (rc != HCA_OK) return rc;
      // paired launches: the wait of the pair's second layer covers the first one's too - layer_done events are
      // recorded in layer order on the attend stream (not so with spare-buffer evictions, whose last slice
      // records it later)
      const bool covered = p->pair && !p->sel_waits && p->d.spare_kcache == nullptr && (l & 1) == 0 &&
                           l + 1 + 2 * S < p->n_layers;
      if (!covered) {
        rc = wait_layer(l + 2 * S);
        if (rc != HCA_OK) return rc;
      }
      nx.b_kcache = layers[l + 2 * S].kcache;
      nx.b_q = layers[l + 2 * S].q;
      nx.b_so = select_view(L, p->d.ws_select[(l + 2 * S) % p->n_sel], mb, k);
    }
    return HCA_OK;
  };
  FusedCtx second;                         // the pair's second layer, until its own turn in the loop
  int second_layer = -1;
  bool have_second = false;
  bool pair_selected = false;              // the pair's second layer already has its selection enqueued
  int pair_selected_layer = -1;
  for (int l = 0; l < p->n_layers; ++l) {
    hca_layer& ly = layers[l];
    int64_t* nl = n_resident + (int64_t)l * L.batch;
    if (ly.kcache == nullptr || ly.acc == nullptr || ly.pos == nullptr || ly.k_new == nullptr || ly.q == nullptr ||
        ly.y == nullptr)
      return HCA_ERR_BAD_ARG;
    if (vq && (ly.vq_centroids == nullptr || ly.vq_lut == nullptr)) return HCA_ERR_BAD_ARG;
    const int s3 = l % p->n_sel, s4 = l % p->n_pipe;
    // where this layer's selection goes: its own buffer, or the one of its set
    const bool own_idx = p->d.layer_idx != nullptr;
    auto idx_of = [&](int l2) -> int32_t* {
      return own_idx ? p->d.layer_idx + (int64_t)l2 * p->d.layer_idx_stride : p->d.idx[l2 % p->n_pipe];
    };
    auto count_of = [&](int l2) -> int32_t* {
      return own_idx ? p->d.layer_count + (int64_t)l2 * L.rows : p->d.count[l2 % p->n_pipe];
    };
    int32_t* const idx_l = idx_of(l);
    int32_t* const count_l = count_of(l);
    const hipStream_t sa = scan_stream(l);           // this layer's scan stream ...
    const hipStream_t sb = p->dual ? sa : sb_topk;   // ... and the stream of its selection
    NRes nr;
    int64_t nmax;
    int32_t rc = HCA_OK;
    // stage 1: append + key scan
    if (fused) {
      if (have_second && second_layer == l) {
        // second layer of a pair: its scan went out with the first layer's, and the top-k stream already waits for it
        nr = second.nr;
        nmax = second.nmax;
        have_second = false;
      } else {
        FusedCtx c0, c1;
        rc = fused_prepare(l, &c0);
        if (rc != HCA_OK) return rc;
        const bool timed = timing_slot >= 0 && l % p->timing_stride == 0;
        if (timed) HCA_HIP(hipEventRecord(p->t0[(size_t)timing_slot * p->n_layers + l], sa));
        hipEvent_t bound = nullptr;
        if (p->pair && l + 1 < p->n_layers) {
          rc = fused_prepare(l + 1, &c1);
          if (rc != HCA_OK) return rc;
          const void* const kc2[2] = {layers[l].kcache, layers[l + 1].kcache};
          const void* const q2[2] = {layers[l].q, layers[l + 1].q};
          const NRes nr2[2] = {c0.nr, c1.nr};
          const int64_t nm2[2] = {c0.nmax, c1.nmax};
          void* const ws2[2] = {p->d.ws_select[s3], p->d.ws_select[(l + 1) % p->n_sel]};
          uint64_t* const st2[2] = {c0.stamps, c1.stamps};
          const SelectStepNext nx2[2] = {c0.nx, c1.nx};
          // the launch's completion event rides on the dispatch itself: the end-of-bracket event when the launch
          // is timed (the selection stream then waits for that one), the layer's score_done otherwise
          bound = timed ? p->t1[(size_t)timing_slot * p->n_layers + l] : (sb != sa ? p->score_done[s3] : nullptr);
          rc = launch_select_scan_step_pair(L, kc2, q2, nr2, nm2, k, ws2, sa, st2, nx2, bound);
          second = c1;
          second_layer = l + 1;
          have_second = true;
        } else {
          rc = launch_select_scan_step(L, ly.kcache, ly.q, c0.nr, c0.nmax, k, p->d.ws_select[s3], sa, c0.stamps, c0.nx);
        }
        if (rc != HCA_OK) return rc;
        if (bound != nullptr) {
          if (sb != sa) HCA_HIP(hipStreamWaitEvent(sb, bound, 0));
        } else {
          if (timed) HCA_HIP(hipEventRecord(p->t1[(size_t)timing_slot * p->n_layers + l], sa));
          if (sb != sa) {
            HCA_HIP(hipEventRecord(p->score_done[s3], sa));
            HCA_HIP(hipStreamWaitEvent(sb, p->score_done[s3], 0));
          }
        }
        nr = c0.nr;
        nmax = c0.nmax;
      }
    } else {
      rc = load_nres(L, nl, &nr, &nmax);
      if (rc != HCA_OK) return rc;
      for (int b = 0; b < L.batch; ++b)
        if (nr.n[b] + 1 > L.cap) return HCA_ERR_CAPACITY;
      const bool timed = timing_slot >= 0 && l % p->timing_stride == 0;
      // top-k of the previous user of this score buffer (with a buffer per layer that is this layer's own
      // previous step, which layer_done covers)
      if (p->sel_waits) HCA_HIP(hipStreamWaitEvent(sa, p->sel_free[s3], 0));
      HCA_HIP(hipStreamWaitEvent(sa, p->layer_done[l], 0));    // this layer's attend / evict of the previous step
      rc = vq ? launch_vq_assign(L, vg, vc, ly.vq_centroids, (uint8_t*)ly.kcache, ly.k_new, 1, nr, ly.acc, ly.pos, vrow0, sa)
              : launch_quantize(L, ly.kcache, ly.k_new, 1, nr, ly.acc, ly.pos, vrow0, sa);
      if (rc != HCA_OK) return rc;
      for (int b = 0; b < L.batch; ++b) { nr.n[b] += 1; nl[b] += 1; }
      nmax += 1;
      if (timed) HCA_HIP(hipEventRecord(p->t0[(size_t)timing_slot * p->n_layers + l], sa));
      uint64_t* stamps = nullptr;
      if (!vq && timing_slot >= 0 && p->d.scan_stamps != nullptr)
        stamps = (uint64_t*)p->d.scan_stamps + ((int64_t)timing_slot * p->n_layers + l) * p->d.scan_stamp_pairs * 2;
      rc = vq ? launch_vq_score(L, vg, vc, ly.vq_centroids, (const uint8_t*)ly.kcache, ly.q, nr, nmax, ly.vq_lut,
                                p->d.sel[s3], nullptr, sa)
              : launch_score(L, ly.kcache, ly.q, nr, nmax, p->d.sel[s3], nullptr, sa, stamps, &p->tune);
      if (rc != HCA_OK) return rc;
      if (timed) HCA_HIP(hipEventRecord(p->t1[(size_t)timing_slot * p->n_layers + l], sa));
      HCA_HIP(hipEventRecord(p->score_done[s3], sa));
      HCA_HIP(hipStreamWaitEvent(sb, p->score_done[s3], 0));
    }
    // stage 2: top-k.  The set of idx / count / staging buffers is free when the layer that used it last is done
    // (its attend, and its eviction if it had one)
    if (pair_selected && pair_selected_layer == l) {
      pair_selected = false;                 // second layer of a pair: selected together with the first
    } else if (fused && have_second && second_layer == l + 1) {
      // first layer of a pair: one selection launch (and one pair of fall-back launches) for both layers
      const int s3b = (l + 1) % p->n_sel, s4b = (l + 1) % p->n_pipe;
      if (!own_idx && p->slot_free[s4] != nullptr) HCA_HIP(hipStreamWaitEvent(sb, p->slot_free[s4], 0));
      if (!own_idx && p->slot_free[s4b] != nullptr) HCA_HIP(hipStreamWaitEvent(sb, p->slot_free[s4b], 0));
      const void* const kc2[2] = {layers[l].kcache, layers[l + 1].kcache};
      const void* const q2[2] = {layers[l].q, layers[l + 1].q};
      const NRes nr2[2] = {nr, second.nr};
      const int64_t nm2[2] = {nmax, second.nmax};
      int32_t* const idx2[2] = {idx_l, idx_of(l + 1)};
      int32_t* const cnt2[2] = {count_l, count_of(l + 1)};
      void* const ws2[2] = {p->d.ws_select[s3], p->d.ws_select[s3b]};
      rc = launch_select_finish_pair(L, kc2, q2, nr2, nm2, k, idx2, cnt2, ws2, sb, p->tune.select_wg == 256);
      if (rc != HCA_OK) return rc;
      if (p->sel_waits) {
        HCA_HIP(hipEventRecord(p->sel_free[s3], sb));
        HCA_HIP(hipEventRecord(p->sel_free[s3b], sb));
      }
      HCA_HIP(hipEventRecord(p->topk_done[s4], sb));
      HCA_HIP(hipEventRecord(p->topk_done[s4b], sb));
      pair_selected = true;
      pair_selected_layer = l + 1;
    } else {
    if (!own_idx && p->slot_free[s4] != nullptr) HCA_HIP(hipStreamWaitEvent(sb, p->slot_free[s4], 0));
    rc = fused ? launch_select_finish(L, ly.kcache, ly.q, nr, nmax, k, idx_l, count_l, p->d.ws_select[s3], sb,
                                      p->tune.select_wg == 256)
         : p->d.topp_tau > 0.0
             ? launch_topp(L, p->d.sel[s3], nr, nmax, sm_scale, p->d.topp_tau, k, idx_l, count_l, nullptr,
                           p->d.ws_topk, sb)
             : launch_topk(L, p->d.sel[s3], nr, nmax, k, idx_l, count_l, p->d.ws_topk, sb, true);
    if (rc != HCA_OK) return rc;
    if (p->sel_waits) HCA_HIP(hipEventRecord(p->sel_free[s3], sb));
    HCA_HIP(hipEventRecord(p->topk_done[s4], sb));
    }
    // stage 3: host-link gather.  With a selection buffer per layer the set of staging buffers is claimed here
    if (own_idx && p->slot_free[s4] != nullptr) HCA_HIP(hipStreamWaitEvent(sg, p->slot_free[s4], 0));
    HCA_HIP(hipStreamWaitEvent(sg, p->topk_done[s4], 0));
    uint64_t* gstamps = nullptr;
    if (timing_slot >= 0 && p->d.gather_stamps != nullptr)
      gstamps = (uint64_t*)p->d.gather_stamps + ((int64_t)timing_slot * p->n_layers + l) * kGatherStampPairs * 2;
    HostShare hs;
    if (hchunks > 0) {
      // hybrid value side: the first chunks of every row's selection are summed by the host threads from the
      // value store itself; what they need (weights relative to each chunk's maximum, value-row numbers)
      // goes out first on this stream, then the signal, then the gather of the remaining entries
      const uint32_t seq = p->host->next_seq();
      hs = p->host->share(s4, seq, p->host_spin_limit);
      hs.chunks = hchunks;
      rc = launch_attend_host_chunks(L, ly.kcache, ly.q, idx_l, count_l, k, ly.pos, n_host_rows, ly.v_hbm,
                                     hbm_stride, sm_scale, p->d.ws_attend[s4], hs, sg);
      if (rc != HCA_OK) return rc;
      p->host->publish(seq, s4, hchunks, ly.v_host, host_stride, n_host_rows);
    }
    rc = launch_gather(L, idx_l, count_l, k, ly.pos, ly.v_host, host_stride, n_host_rows, ly.v_hbm,
                       hbm_stride, p->d.ws_attend[s4], sg, gstamps, hchunks * kAttendChunk, &p->tune,
                       hchunks > 0 ? &hs : nullptr);
    if (rc != HCA_OK) return rc;
    HCA_HIP(hipEventRecord(p->gather_done[s4], sg));
    // stage 4: attend (+ eviction into the spare buffers, which then swap with the layer's)
    HCA_HIP(hipStreamWaitEvent(sc, p->gather_done[s4], 0));
    rc = vq ? launch_vq_attend_gathered(L, vg, vc, (const uint8_t*)ly.kcache, ly.vq_lut, idx_l, count_l, k,
                                        sm_scale, ly.y, ly.acc, p->d.ws_attend[s4], sc)
            : launch_attend_gathered(L, ly.kcache, ly.q, idx_l, count_l, k, sm_scale, ly.y, ly.acc,
                                     p->d.ws_attend[s4], sc, nullptr, hchunks > 0 ? &hs : nullptr);
    if (rc != HCA_OK) return rc;
    const int64_t M = evict_M != nullptr ? evict_M[l] : 0;
    bool starts_job = false;
    if (M != 0) {
      bool any = false;
      for (int b = 0; b < L.batch; ++b) any = any || nr.n[b] > M;
      if (any && p->d.spare_kcache == nullptr) {
        // no spare buffers: compact in place behind this attend.  Rows below the first dropped slot keep
        // their place, so when the dropped tokens sit near the end (the usual case: ties go against the
        // higher slot) only the select passes and a short tail move are paid
        rc = vq ? launch_vq_evict(L, vg, vc, (uint8_t*)ly.kcache, ly.acc, ly.pos, nr, nmax, M, n_protect, nullptr,
                                  p->d.ws_evict, nullptr, nullptr, nullptr, sc)
                : launch_evict(L, ly.kcache, ly.acc, ly.pos, nr, nmax, M, n_protect, nullptr, p->d.ws_evict, nullptr,
                               nullptr, nullptr, sc);
        if (rc != HCA_OK) return rc;
        for (int b = 0; b < L.batch; ++b) if (nl[b] > M) nl[b] = M;
      } else if (any) {
        // one spare set: finish a job still in flight before the next one starts
        while (job.active) {
          rc = advance(job);
          if (rc != HCA_OK) return rc;
        }
        job.active = true; job.layer = l; job.next_slice = 0; job.nr = nr; job.nmax = nmax; job.M = M;
        starts_job = true;
        HCA_HIP(hipEventRecord(p->pipe_free[s4], sc));     // the set is free now; layer_done comes with the last slice
        for (int b = 0; b < L.batch; ++b) if (nl[b] > M) nl[b] = M;
      }
    }
    if (job.active) {                      // one slice of the eviction in flight rides behind this attend
      rc = advance(job);
      if (rc != HCA_OK) return rc;
    }
    if (!starts_job) {
      HCA_HIP(hipEventRecord(p->layer_done[l], sc));
      p->slot_free[s4] = p->layer_done[l];
    } else {                               // the job's last slice records layer_done
      p->slot_free[s4] = p->pipe_free[s4];
    }
  }
  while (job.active) {                     // the step ends with every started eviction fully enqueued
    int32_t rc = advance(job);
    if (rc != HCA_OK) return rc;
  }
  return HCA_OK;
}

int32_t hca_pipeline_host_status(hca_pipeline* p, uint32_t* wait_timeouts, uint32_t* bad_rows, double* mean_job_us,
                                 double* mean_chunk_us) {
  if (p == nullptr) return HCA_ERR_BAD_ARG;
  if (wait_timeouts != nullptr) *wait_timeouts = p->host ? p->host->errors() : 0u;
  if (bad_rows != nullptr) *bad_rows = p->host ? p->host->bad_rows() : 0u;
  double ju = 0.0, tu = 0.0;
  if (p->host) p->host->times(&ju, &tu);
  if (mean_job_us != nullptr) *mean_job_us = ju;
  if (mean_chunk_us != nullptr) *mean_chunk_us = tu;
  return HCA_OK;
}

int64_t hca_scan_stamp_pairs(const hca_shape* shape, int64_t n_tokens) {
  Layout L;
  if (make_layout(shape, &L) != HCA_OK || n_tokens < 0) return 0;
  return score_stamp_pairs(L, n_tokens);
}

int32_t hca_wall_clock_khz(void) {
  int dev = 0, khz = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess) return 0;
  return khz;
}

int32_t hca_pipeline_scan_ms(hca_pipeline* p, int32_t timing_slot, float* ms) {
  if (p == nullptr || ms == nullptr || timing_slot < 0 || timing_slot >= p->timing_slots) return HCA_ERR_BAD_ARG;
  for (int l = 0; l < p->n_layers; ++l) {
    const size_t i = (size_t)timing_slot * p->n_layers + l;
    ms[l] = -1.0f;                                    // layers without a bracket
    // (paired launches: the bracket of an even layer holds the launch it shares with the next layer)
    if (l % p->timing_stride == 0 && !(p->pair && (l & 1))) HCA_HIP(hipEventElapsedTime(&ms[l], p->t0[i], p->t1[i]));
  }
  return HCA_OK;
}

}  // extern "C"
