// The host half of the paper's CPU-GPU split (Sec. 3.2 "CPU part", Eq. 5): the GPU hands over, per selected
// token, its value-row number and one 2-byte weight per query head (hca_attend_weights); the host forms
// y = sum_i w_i V_i from the value store that never leaves host memory.  Host code only.
#include <immintrin.h>
#include <unistd.h>

#include <atomic>
#include <chrono>
#include <cmath>
#include <condition_variable>
#include <cstring>
#include <functional>
#include <memory>
#include <mutex>
#include <thread>
#include <vector>

#include "hca_internal.h"

namespace hca {

static inline float half_to_float(uint16_t h) {
  _Float16 v;
  std::memcpy(&v, &h, 2);
  return (float)v;
}

// y_part[G][128] += sum over selected tokens [i0, i1) of one row
[[maybe_unused]] static void sum_range_plain(int G, int32_t k, const int32_t* vrow, const uint16_t* w /*[G][k]*/, const uint16_t* v_row0,
                            int64_t i0, int64_t i1, float* y_part) {
  for (int64_t i = i0; i < i1; ++i) {
    const int32_t r = vrow[i];
    if (r < 0) continue;
    const _Float16* v = reinterpret_cast<const _Float16*>(v_row0) + (int64_t)r * kHeadDim;
    if (i + 4 < i1 && vrow[i + 4] >= 0)            // the rows are scattered: ask for one ahead
      __builtin_prefetch(v_row0 + (int64_t)vrow[i + 4] * kHeadDim);
    float vf[kHeadDim];
    for (int c = 0; c < kHeadDim; ++c) vf[c] = (float)v[c];
    for (int h = 0; h < G; ++h) {
      const float wh = half_to_float(w[(int64_t)h * k + i]);
      float* __restrict__ y = y_part + h * kHeadDim;
      for (int c = 0; c < kHeadDim; ++c) y[c] += wh * vf[c];
    }
  }
}

#if defined(__AVX2__) && defined(__FMA__) && defined(__F16C__)
// The same with 8-wide fp16 -> fp32 conversion and fused multiply-adds (the host pass of this library is built
// with these instruction sets switched on).  Per output element the terms are added in the same order as above.
static void sum_range_avx2(int G, int32_t k, const int32_t* vrow,
                                                                    const uint16_t* w, const uint16_t* v_row0,
                                                                    int64_t i0, int64_t i1, float* y_part) {
  constexpr int kAhead = 8;                        // rows asked for ahead of use (each row is four cache lines)
  for (int64_t i = i0; i < i1; ++i) {
    const int32_t r = vrow[i];
    if (r < 0) continue;
    if (i + kAhead < i1 && vrow[i + kAhead] >= 0) {
      const char* nx = reinterpret_cast<const char*>(v_row0 + (int64_t)vrow[i + kAhead] * kHeadDim);
      _mm_prefetch(nx, _MM_HINT_T0);
      _mm_prefetch(nx + 64, _MM_HINT_T0);
      _mm_prefetch(nx + 128, _MM_HINT_T0);
      _mm_prefetch(nx + 192, _MM_HINT_T0);
    }
    const __m128i* v = reinterpret_cast<const __m128i*>(v_row0 + (int64_t)r * kHeadDim);
    __m256 vf[kHeadDim / 8];
    for (int c = 0; c < kHeadDim / 8; ++c) vf[c] = _mm256_cvtph_ps(_mm_loadu_si128(v + c));
    for (int h = 0; h < G; ++h) {
      const __m256 wh = _mm256_set1_ps(half_to_float(w[(int64_t)h * k + i]));
      float* y = y_part + h * kHeadDim;
      for (int c = 0; c < kHeadDim / 8; ++c)
        _mm256_storeu_ps(y + 8 * c, _mm256_fmadd_ps(wh, vf[c], _mm256_loadu_ps(y + 8 * c)));
    }
  }
}

constexpr auto sum_range = sum_range_avx2;
#else
constexpr auto sum_range = sum_range_plain;
#endif

#if defined(__x86_64__)
// AVX-512 form of host_chunk_sum (chosen at run time when the CPU has it; this translation unit is built for
// AVX2).  Two passes over the chunk's rows, one per 128-byte half of a value row (64 channels): the partial sums
// of the four query heads for those 64 channels stay in 16 registers for the whole pass, so a token costs one
// conversion and four multiply-adds per 16 channels and no traffic to the accumulators.  The halves are
// different cache lines, so nothing is fetched twice; rows are asked for well ahead of use.
__attribute__((target("avx512f,avx512vl,avx512bw,f16c,fma"))) static int chunk_sum_avx512(
    int G, const float* p, const int32_t* vrow, const uint16_t* v_row0, int64_t n_rows, float* py) {
  constexpr int kAhead = 24;
  int bad = 0;
  for (int half = 0; half < 2; ++half) {
    __m512 acc[4][4];
    for (int h = 0; h < 4; ++h)
      for (int c = 0; c < 4; ++c) acc[h][c] = _mm512_setzero_ps();
    const uint16_t* base = v_row0 + half * 64;
    for (int i = 0; i < kAttendChunk; ++i) {
      if (i + kAhead < kAttendChunk) {
        const int32_t rn = vrow[i + kAhead];
        if (rn >= 0 && rn < n_rows) {
          const char* nx = reinterpret_cast<const char*>(base + (int64_t)rn * kHeadDim);
          _mm_prefetch(nx, _MM_HINT_T0);
          _mm_prefetch(nx + 64, _MM_HINT_T0);
        }
      }
      const int32_t r = vrow[i];
      if (r < 0) continue;
      if (r >= n_rows) { bad += half == 0; continue; }
      const __m256i* v = reinterpret_cast<const __m256i*>(base + (int64_t)r * kHeadDim);
      __m512 vf[4];
      for (int c = 0; c < 4; ++c) vf[c] = _mm512_cvtph_ps(_mm256_loadu_si256(v + c));
      for (int h = 0; h < G; ++h) {
        const __m512 wh = _mm512_set1_ps(p[h * kAttendChunk + i]);
        for (int c = 0; c < 4; ++c) acc[h][c] = _mm512_fmadd_ps(wh, vf[c], acc[h][c]);
      }
    }
    for (int h = 0; h < 4; ++h)
      for (int c = 0; c < 4; ++c) _mm512_storeu_ps(py + h * kHeadDim + half * 64 + 16 * c, acc[h][c]);
  }
  return bad;
}
#endif

// One chunk of the host share of a decode step (the step driver's worker threads call this): fp32 weights
// p[h][i] (relative to the chunk's maximum; the GPU merges the chunks), value rows read where they live.
int host_chunk_sum(int G, const float* p, const int32_t* vrow, const uint16_t* v_row0, int64_t n_rows, float* py) {
#if defined(__x86_64__)
  static const bool has512 = __builtin_cpu_supports("avx512f") && __builtin_cpu_supports("avx512vl") &&
                             __builtin_cpu_supports("avx512bw");
  if (has512 && tuning().host_isa != 2) return chunk_sum_avx512(G, p, vrow, v_row0, n_rows, py);
#endif
  alignas(64) float acc[4 * kHeadDim];
  std::memset(acc, 0, sizeof(acc));
  int bad = 0;
#if defined(__AVX2__) && defined(__FMA__) && defined(__F16C__)
  constexpr int kAhead = 8;
  for (int i = 0; i < kAttendChunk; ++i) {
    const int32_t r = vrow[i];
    if (i + kAhead < kAttendChunk) {
      const int32_t rn = vrow[i + kAhead];
      if (rn >= 0 && rn < n_rows) {
        const char* nx = reinterpret_cast<const char*>(v_row0 + (int64_t)rn * kHeadDim);
        _mm_prefetch(nx, _MM_HINT_T0);
        _mm_prefetch(nx + 64, _MM_HINT_T0);
        _mm_prefetch(nx + 128, _MM_HINT_T0);
        _mm_prefetch(nx + 192, _MM_HINT_T0);
      }
    }
    if (r < 0) continue;
    if (r >= n_rows) { ++bad; continue; }
    const __m128i* v = reinterpret_cast<const __m128i*>(v_row0 + (int64_t)r * kHeadDim);
    __m256 vf[kHeadDim / 8];
    for (int c = 0; c < kHeadDim / 8; ++c) vf[c] = _mm256_cvtph_ps(_mm_loadu_si128(v + c));
    for (int h = 0; h < G; ++h) {
      const __m256 wh = _mm256_set1_ps(p[h * kAttendChunk + i]);
      float* y = acc + h * kHeadDim;
      for (int c = 0; c < kHeadDim / 8; ++c)
        _mm256_store_ps(y + 8 * c, _mm256_fmadd_ps(wh, vf[c], _mm256_load_ps(y + 8 * c)));
    }
  }
#else
  for (int i = 0; i < kAttendChunk; ++i) {
    const int32_t r = vrow[i];
    if (r < 0) continue;
    if (r >= n_rows) { ++bad; continue; }
    const _Float16* v = reinterpret_cast<const _Float16*>(v_row0) + (int64_t)r * kHeadDim;
    for (int h = 0; h < G; ++h) {
      const float wh = p[h * kAttendChunk + i];
      for (int c = 0; c < kHeadDim; ++c) acc[h * kHeadDim + c] = fmaf(wh, (float)v[c], acc[h * kHeadDim + c]);
    }
  }
#endif
  std::memcpy(py, acc, sizeof(float) * 4 * kHeadDim);
  return bad;
}

// Worker threads that outlive the call: starting sixteen threads costs more than the sum they are started for.
// One job at a time (callers are serialised); the calling thread works along and the call ends when the last
// task has ended, whoever ran it: a worker that wakes late finds its job drained and goes back to waiting,
// nobody waits for it.  The threads are never joined: they sleep on the condition variable until the process ends.
class HostPool {
 public:
  static HostPool& get() {
    // never destroyed: the workers may outlive static destructors.  A forked child inherits the object but none
    // of its threads, so it starts a pool of its own.
    static std::mutex mu;
    static HostPool* p = nullptr;
    static pid_t owner = 0;
    std::lock_guard<std::mutex> g(mu);
    const pid_t me = getpid();
    if (p == nullptr || owner != me) {
      p = new HostPool();
      owner = me;
    }
    return *p;
  }
  template <class F>
  void run(int n_threads, int ntask, F&& task) {
    std::lock_guard<std::mutex> serial(call_);
    grow(n_threads - 1);
    auto job = std::make_shared<Job>();
    job->fn = [&](int t) { task(t); };
    job->ntask = ntask;
    job->helpers = n_threads - 1;
    {
      std::lock_guard<std::mutex> g(m_);
      job_ = job;
      generation_.store(generation_.load(std::memory_order_relaxed) + 1, std::memory_order_release);
    }
    cv_.notify_all();
    drain(*job);
    // the tasks still running on other threads: short ones, so poll
    while (job->finished.load(std::memory_order_acquire) < ntask) _mm_pause();
  }

 private:
  // One call's work.  Workers hold it by shared pointer, so one that is still looking at it when the call
  // has returned touches memory that is still there - and, every task having been claimed, nothing else.
  struct Job {
    std::function<void(int)> fn;
    int ntask = 0, helpers = 0;
    std::atomic<int> next{0}, finished{0};
  };
  static void drain(Job& j) {
    for (int t = j.next.fetch_add(1); t < j.ntask; t = j.next.fetch_add(1)) {
      j.fn(t);
      j.finished.fetch_add(1, std::memory_order_release);
    }
  }
  void grow(int want) {
    while ((int)workers_.size() < want) {
      const int id = (int)workers_.size();
      workers_.emplace_back([this, id] { loop(id); });
      workers_.back().detach();
    }
  }
  void loop(int id) {
    uint64_t seen = 0;
    for (;;) {
      // a decode loop calls again within a fraction of a millisecond: poll for that long before sleeping
      const auto t0 = std::chrono::steady_clock::now();
      while (generation_.load(std::memory_order_acquire) == seen) {
        for (int i = 0; i < 64; ++i) _mm_pause();
        if (std::chrono::steady_clock::now() - t0 >= std::chrono::microseconds(tuning().host_spin_us)) break;
      }
      std::shared_ptr<Job> job;
      {
        std::unique_lock<std::mutex> g(m_);
        cv_.wait(g, [&] { return generation_.load(std::memory_order_relaxed) != seen; });
        seen = generation_.load(std::memory_order_relaxed);
        job = job_;
      }
      if (id < job->helpers) drain(*job);           // else this job asked for fewer threads
    }
  }
  std::mutex call_, m_;
  std::condition_variable cv_;
  std::vector<std::thread> workers_;
  std::shared_ptr<Job> job_;
  std::atomic<uint64_t> generation_{0};
};

}  // namespace hca

using namespace hca;

extern "C" int32_t hca_host_weighted_sum(const hca_shape* shape, const int32_t* vrow, const int32_t* count, int32_t k,
                                         const void* w_f16, const void* v_host, int64_t host_stride, float* y,
                                         int32_t n_threads) {
  Layout L;
  hca_shape s;
  if (shape == nullptr) return HCA_ERR_BAD_ARG;
  s = *shape;
  s.bits = 4;
  s.group = 32;                                   // the code format plays no part on the host side
  int32_t rc = make_layout(&s, &L);
  if (rc != HCA_OK) return rc;
  if (vrow == nullptr || count == nullptr || w_f16 == nullptr || v_host == nullptr || y == nullptr) return HCA_ERR_BAD_ARG;
  if (k < 1 || host_stride < 1) return HCA_ERR_BAD_ARG;
  if (n_threads < 1) n_threads = 1;
  if (n_threads > 64) n_threads = 64;
  const int G = L.gqa;
  // tasks: every row cut into `parts` ranges of its selected tokens, partial sums added up afterwards
  // (four tasks per thread when there are several threads: the threads do not all start at the same moment)
  int parts = ((n_threads > 1 ? 4 * n_threads : 1) + L.rows - 1) / L.rows;
  if (parts < 1) parts = 1;
  const int ntask = L.rows * parts;
  for (int row = 0; row < L.rows; ++row) {
    int64_t cnt = count[row] < k ? count[row] : k;
    for (int64_t i = 0; i < cnt; ++i)
      if (vrow[(int64_t)row * k + i] >= host_stride) return HCA_ERR_CAPACITY;
  }
  std::vector<float> partial((size_t)ntask * G * kHeadDim, 0.0f);
  auto task = [&](int t) {
    const int row = t / parts, part = t % parts;
    int64_t cnt = count[row];
    if (cnt > k) cnt = k;
    const int64_t per = (cnt + parts - 1) / parts;
    int64_t i0 = per * part, i1 = i0 + per;
    if (i1 > cnt) i1 = cnt;
    if (i0 >= i1) return;
    // the running sums live on the stack of the thread that forms them and are handed over once at the end
    alignas(64) float acc[4 * kHeadDim];             // at most four query heads share a KV head
    std::memset(acc, 0, sizeof(float) * G * kHeadDim);
    sum_range(G, k, vrow + (int64_t)row * k, (const uint16_t*)w_f16 + (int64_t)row * G * k,
              (const uint16_t*)v_host + (int64_t)row * host_stride * kHeadDim, i0, i1, acc);
    std::memcpy(&partial[(size_t)t * G * kHeadDim], acc, sizeof(float) * G * kHeadDim);
  };
  if (n_threads == 1) {
    for (int t = 0; t < ntask; ++t) task(t);
  } else {
    HostPool::get().run(n_threads, ntask, task);
  }
  for (int row = 0; row < L.rows; ++row)
    for (int e = 0; e < G * kHeadDim; ++e) {
      float acc = 0.0f;
      for (int part = 0; part < parts; ++part) acc += partial[((size_t)row * parts + part) * G * kHeadDim + e];
      y[(int64_t)row * G * kHeadDim + e] = acc;
    }
  return HCA_OK;
}

// The first CPU access to each 4 KiB page of a pinned allocation is a page fault (the pages exist and are
// pinned, but the CPU's own mapping of them is made on demand; microseconds each, and the handlers of several
// threads serialise).  A value store that host threads will read at random rows is therefore walked once,
// one byte per page, before the first decode step.
extern "C" int32_t hca_host_prefault(const void* ptr, size_t bytes, int32_t n_threads) {
  if (ptr == nullptr && bytes != 0) return HCA_ERR_BAD_ARG;
  if (n_threads < 1) n_threads = 1;
  if (n_threads > 64) n_threads = 64;
  constexpr size_t kPage = 4096;
  const size_t pages = (bytes + kPage - 1) / kPage;
  const unsigned char* base = (const unsigned char*)ptr;
  auto walk = [&](size_t p0, size_t p1) {
    unsigned sum = 0;
    for (size_t p = p0; p < p1; ++p) sum += *(const volatile unsigned char*)(base + p * kPage);
    (void)sum;
  };
  std::vector<std::thread> th;
  const size_t per = (pages + n_threads - 1) / n_threads;
  for (int t = 1; t < n_threads; ++t) {
    const size_t p0 = per * t, p1 = p0 + per < pages ? p0 + per : pages;
    if (p0 < p1) th.emplace_back(walk, p0, p1);
  }
  walk(0, per < pages ? per : pages);
  for (auto& t : th) t.join();
  return HCA_OK;
}

// Test / debug: one chunk of the hybrid value side's host work (what a worker thread of the step driver does).
extern "C" int32_t hca_debug_host_chunk_sum(int32_t gqa, const float* p, const int32_t* vrow, const void* v_rows,
                                            int64_t n_rows, float* py) {
  if (gqa < 1 || gqa > 4 || p == nullptr || vrow == nullptr || v_rows == nullptr || py == nullptr || n_rows < 0)
    return HCA_ERR_BAD_ARG;
  return host_chunk_sum(gqa, p, vrow, (const uint16_t*)v_rows, n_rows, py);
}

