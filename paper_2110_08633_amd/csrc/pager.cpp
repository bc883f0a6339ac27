// Staging tier of the swap engine for host state that is NOT page-locked.
//
// The method keeps every model's state in host DRAM (paper Section 2.3); the
// copy engines and the library's copy kernel can only reach page-locked
// memory, and how much of that a process may hold is limited by the driver
// (64 GiB on the machines this was developed on, next to 300 GB of DRAM).
// Models whose arrays do not fit are therefore given ordinary memory, and
// their promotes and write-backs travel through a small page-locked ring the
// caller provides:
//
//   promote   pageable array -> (host threads, memcpy) -> ring chunk
//             -> (SDMA, h2d stream) -> shard buffer
//   demote    shard buffer -> (copy kernel or SDMA, d2h stream) -> ring chunk
//             -> (host threads, memcpy) -> pageable array
//
// One coordinator thread per direction runs the jobs of its direction in the
// order they were submitted (so each copy stream sees its operations in
// program order) and a few helper threads share every chunk's memcpy; several
// ring chunks are in flight so that memcpy and link transfer overlap.  The
// calling thread never copies: it submits a job and gets a ticket; whoever
// depends on the job having been ISSUED to the stream (an event recorded by it)
// waits for the ticket first.
#include <immintrin.h>

#include <atomic>
#include <chrono>
#include <condition_variable>
#include <cstring>
#include <deque>
#include <functional>
#include <mutex>
#include <thread>

#include "hydra_internal.h"

namespace hydra {

// fp32 -> bf16, round to nearest even (NaN stays NaN): bit for bit what the device's casts produce
static void round_bf16_plain(uint16_t *dst, const float *src, size_t n) {
  for (size_t i = 0; i < n; ++i) {
    uint32_t u;
    memcpy(&u, src + i, 4);
    const uint32_t r = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    dst[i] = (uint16_t)((u & 0x7fffffffu) > 0x7f800000u ? ((u >> 16) | 0x40u) : r);
  }
}

// the same, 16 values per step (the write-back path of the staging tier rounds a third of all bytes it moves: the
// plain loop halved what a helper thread moves per second)
__attribute__((target("avx2"))) static inline __m256i round8_avx2(const float *p) {
  const __m256i u = _mm256_loadu_si256((const __m256i *)p);
  const __m256i hi = _mm256_srli_epi32(u, 16);
  const __m256i r = _mm256_srli_epi32(
      _mm256_add_epi32(_mm256_add_epi32(u, _mm256_set1_epi32(0x7fff)), _mm256_and_si256(hi, _mm256_set1_epi32(1))), 16);
  // both sides of the comparison are below 2^31: the signed one does
  const __m256i nan = _mm256_cmpgt_epi32(_mm256_and_si256(u, _mm256_set1_epi32(0x7fffffff)), _mm256_set1_epi32(0x7f800000));
  return _mm256_blendv_epi8(r, _mm256_or_si256(hi, _mm256_set1_epi32(0x40)), nan);
}

__attribute__((target("avx2"))) static void round_bf16_avx2(uint16_t *dst, const float *src, size_t n) {
  size_t i = 0;
  for (; i + 16 <= n; i += 16) {
    // the pack works per 128-bit half (a0-3 b0-3 | a4-7 b4-7): the permutation restores the order
    const __m256i p = _mm256_packus_epi32(round8_avx2(src + i), round8_avx2(src + i + 8));
    _mm256_storeu_si256((__m256i *)(dst + i), _mm256_permute4x64_epi64(p, 0xD8));
  }
  round_bf16_plain(dst + i, src + i, n - i);
}

void host_round_bf16(uint16_t *dst, const float *src, size_t n) {
  static const bool avx2 = __builtin_cpu_supports("avx2");
  if (avx2) round_bf16_avx2(dst, src, n);
  else round_bf16_plain(dst, src, n);
}

void host_round_bf16_threads(uint16_t *dst, const float *src, size_t n, int threads) {
  if (threads < 1) threads = 1;
  if (n < ((size_t)1 << 22)) threads = 1;
  const size_t per = (n + threads - 1) / threads;
  std::vector<std::thread> th;
  for (int t = 1; t < threads; ++t) {
    const size_t lo = per * t, hi = lo + per < n ? lo + per : n;
    if (lo < hi) th.emplace_back([=] { host_round_bf16(dst + lo, src + lo, hi - lo); });
  }
  host_round_bf16(dst, src, per < n ? per : n);
  for (std::thread &t : th) t.join();
}

// A thread of the library's own that runs host-side jobs in submission order (the rounding of a written-back
// page-locked master into the host's bf16 copy).
struct HostWorker {
  std::thread th;
  std::mutex mu;
  std::condition_variable cv, progress;
  std::deque<std::function<void()>> q;
  uint64_t submitted = 0, executed = 0;
  bool stop = false;
};

hipError_t wait_event(hydra_ctx *ctx, hipEvent_t e) {
  if (!ctx->gate_on) return hipEventSynchronize(e);
  for (;;) {
    hipError_t r;
    {
      HipGate g(ctx);
      r = hipEventQuery(e);
    }
    if (r != hipErrorNotReady) return r;
    std::this_thread::sleep_for(std::chrono::microseconds(20));
  }
}

HostWorker *worker_create() {
  HostWorker *w = new HostWorker();
  w->th = std::thread([w] {
    for (;;) {
      std::function<void()> job;
      {
        std::unique_lock<std::mutex> l(w->mu);
        w->cv.wait(l, [&] { return w->stop || !w->q.empty(); });
        if (w->q.empty()) return;
        job = std::move(w->q.front());
        w->q.pop_front();
      }
      job();
      {
        std::lock_guard<std::mutex> l(w->mu);
        ++w->executed;
      }
      w->progress.notify_all();
    }
  });
  return w;
}

void worker_destroy(HostWorker *w) {
  if (!w) return;
  {
    std::lock_guard<std::mutex> l(w->mu);
    w->stop = true;
  }
  w->cv.notify_all();
  if (w->th.joinable()) w->th.join();  // runs what is still queued first
  delete w;
}

uint64_t worker_submit(HostWorker *w, std::function<void()> job) {
  uint64_t ticket;
  {
    std::lock_guard<std::mutex> l(w->mu);
    w->q.push_back(std::move(job));
    ticket = ++w->submitted;
  }
  w->cv.notify_one();
  return ticket;
}

void worker_wait(HostWorker *w, uint64_t ticket) {
  std::unique_lock<std::mutex> l(w->mu);
  w->progress.wait(l, [&] { return w->executed >= ticket; });
}

void worker_drain(HostWorker *w) {
  std::unique_lock<std::mutex> l(w->mu);
  w->progress.wait(l, [&] { return w->executed >= w->submitted; });
}

namespace {

// one part of a chunk: copied, and (rounded != null) its floats also rounded to bf16 while they are in the cache
inline void copy_part(char *dst, const char *src, size_t n, uint16_t *rounded) {
  if (!rounded) {
    memcpy(dst, src, n);
    return;
  }
  const size_t blk = 1u << 16;  // bytes
  for (size_t o = 0; o < n; o += blk) {
    const size_t c = n - o < blk ? n - o : blk;
    memcpy(dst + o, src + o, c);
    host_round_bf16(rounded + o / 4, (const float *)(src + o), c / 4);
  }
}

// n bytes copied by the calling thread and a few helpers, each a contiguous part; with 'rounded' the bytes are floats
// whose bf16 roundings go to rounded[0 .. n/4)
class CopyPool {
 public:
  explicit CopyPool(int helpers) {
    for (int i = 0; i < helpers; ++i) th_.emplace_back([this, i] { run(i); });
  }
  ~CopyPool() {
    {
      std::lock_guard<std::mutex> l(mu_);
      stop_ = true;
    }
    cv_.notify_all();
    for (std::thread &t : th_) t.join();
  }
  void copy(void *dst, const void *src, size_t n, uint16_t *rounded = nullptr) {
    const size_t parts = th_.size() + 1;
    if (n < (1u << 20) || parts == 1) {
      copy_part((char *)dst, (const char *)src, n, rounded);
      return;
    }
    const size_t per = (n / parts + 4095) & ~(size_t)4095;
    {
      std::lock_guard<std::mutex> l(mu_);
      dst_ = (char *)dst; src_ = (const char *)src; n_ = n; per_ = per; rounded_ = rounded;
      pending_ = (int)th_.size();
      ++gen_;
    }
    cv_.notify_all();
    copy_part((char *)dst, (const char *)src, per < n ? per : n, rounded);  // part 0
    std::unique_lock<std::mutex> l(mu_);
    done_.wait(l, [this] { return pending_ == 0; });
  }

 private:
  void run(int i) {
    uint64_t seen = 0;
    for (;;) {
      std::unique_lock<std::mutex> l(mu_);
      cv_.wait(l, [&] { return stop_ || gen_ != seen; });
      if (stop_) return;
      seen = gen_;
      const size_t lo = per_ * (size_t)(i + 1);
      const size_t hi = lo + per_ < n_ ? lo + per_ : n_;
      char *d = dst_;
      const char *s = src_;
      uint16_t *r = rounded_;
      l.unlock();
      if (lo < hi) copy_part(d + lo, s + lo, hi - lo, r ? r + lo / 4 : nullptr);
      l.lock();
      if (--pending_ == 0) done_.notify_one();
    }
  }
  std::vector<std::thread> th_;
  std::mutex mu_;
  std::condition_variable cv_, done_;
  bool stop_ = false;
  uint64_t gen_ = 0;
  char *dst_ = nullptr;
  const char *src_ = nullptr;
  uint16_t *rounded_ = nullptr;
  size_t n_ = 0, per_ = 0;
  int pending_ = 0;
};

struct Ring {
  char *host = nullptr;    // page-locked
  char *mapped = nullptr;  // the same memory as the device sees it
  size_t chunk = 0;
  int n = 0;
  std::vector<hipEvent_t> ev;  // per chunk: last operation of the copy stream that touched it
  std::vector<char> used;
  uint64_t next = 0;
  int small_k = -1;      // promotes: the chunk that collects copies of less than 1 MiB (-1: none), and how much of
  size_t small_off = 0;  // it they have taken
};

struct Queue {
  std::thread th;
  std::mutex mu;
  std::condition_variable cv, progress;
  std::deque<std::function<hydra_status()>> q;
  uint64_t submitted = 0, executed = 0;
  bool stop = false;
};

}  // namespace

struct Pager {
  hydra_ctx *ctx = nullptr;
  Ring ring[2];
  Queue queue[2];
  CopyPool *pool[2] = {nullptr, nullptr};
  std::mutex err_mu;
  hydra_status err = HYDRA_OK;
  std::string err_text;
};

static void pager_fail(Pager *p, hydra_status st, const std::string &text) {
  std::lock_guard<std::mutex> l(p->err_mu);
  if (p->err == HYDRA_OK) {
    p->err = st;
    p->err_text = text;
  }
}

static void queue_loop(Pager *p, int which) {
  Queue &Q = p->queue[which];
  for (;;) {
    std::function<hydra_status()> job;
    {
      std::unique_lock<std::mutex> l(Q.mu);
      Q.cv.wait(l, [&] { return Q.stop || !Q.q.empty(); });
      if (Q.q.empty()) return;  // stop requested and nothing left
      job = std::move(Q.q.front());
      Q.q.pop_front();
    }
    bool failed;
    {
      std::lock_guard<std::mutex> l(p->err_mu);
      failed = p->err != HYDRA_OK;
    }
    if (!failed) {  // after an error the remaining jobs are dropped (their tickets still advance)
      const hydra_status st = job();
      if (st != HYDRA_OK) pager_fail(p, st, which == PQ_H2D ? "staged promote failed" : "staged write-back failed");
    }
    {
      std::lock_guard<std::mutex> l(Q.mu);
      ++Q.executed;
    }
    Q.progress.notify_all();
  }
}

Pager *pager_create(hydra_ctx *ctx, void *stage, uint64_t stage_bytes, int helpers, std::string *err) {
  if (!stage) {  // no staging area: the two coordinator threads only issue what goes straight to page-locked memory
    Pager *p = new Pager();
    p->ctx = ctx;
    for (int w = 0; w < 2; ++w) p->queue[w].th = std::thread(queue_loop, p, w);
    return p;
  }
  hipPointerAttribute_t at;
  if (hipPointerGetAttributes(&at, stage) != hipSuccess || at.type != hipMemoryTypeHost || !at.devicePointer) {
    (void)hipGetLastError();
    *err = "the staging area is not page-locked host memory";
    return nullptr;
  }
  if (((uintptr_t)stage & 255) || ((uintptr_t)at.devicePointer & 255)) {
    *err = "the staging area must be 256-byte aligned";
    return nullptr;
  }
  // each direction gets half of the area as a ring of up to 8 chunks of at most 64 MiB (multiples of 1 MiB)
  const uint64_t half = stage_bytes / 2;
  uint64_t chunk = (half / 8) & ~((uint64_t)(1 << 20) - 1);
  if (chunk > (64u << 20)) chunk = 64u << 20;
  if (chunk < (1u << 20)) {
    *err = "the staging area must hold at least 16 MiB";
    return nullptr;
  }
  Pager *p = new Pager();
  p->ctx = ctx;
  for (int w = 0; w < 2; ++w) {
    Ring &r = p->ring[w];
    r.host = (char *)stage + w * half;
    r.mapped = (char *)at.devicePointer + w * half;
    r.chunk = chunk;
    r.n = (int)(half / chunk);
    if (r.n > 8) r.n = 8;
    r.ev.assign(r.n, nullptr);
    r.used.assign(r.n, 0);
    for (hipEvent_t &e : r.ev)
      if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) {
        *err = "cannot create the staging ring's events";
        pager_destroy(p);
        return nullptr;
      }
    p->pool[w] = new CopyPool(helpers);
  }
  for (int w = 0; w < 2; ++w) p->queue[w].th = std::thread(queue_loop, p, w);
  return p;
}

void pager_destroy(Pager *p) {
  if (!p) return;
  for (int w = 0; w < 2; ++w) {
    Queue &Q = p->queue[w];
    {
      std::lock_guard<std::mutex> l(Q.mu);
      Q.stop = true;
    }
    Q.cv.notify_all();
    if (Q.th.joinable()) Q.th.join();
  }
  for (int w = 0; w < 2; ++w) {
    delete p->pool[w];
    for (hipEvent_t e : p->ring[w].ev)
      if (e) (void)hipEventDestroy(e);
  }
  delete p;
}

uint64_t pager_submit(Pager *p, int which, std::function<hydra_status()> job) {
  Queue &Q = p->queue[which];
  uint64_t ticket;
  {
    std::lock_guard<std::mutex> l(Q.mu);
    Q.q.push_back(std::move(job));
    ticket = ++Q.submitted;
  }
  Q.cv.notify_one();
  return ticket;
}

void pager_wait(Pager *p, int which, uint64_t ticket) {
  Queue &Q = p->queue[which];
  std::unique_lock<std::mutex> l(Q.mu);
  Q.progress.wait(l, [&] { return Q.executed >= ticket; });
}

hydra_status pager_error(Pager *p, std::string *text) {
  std::lock_guard<std::mutex> l(p->err_mu);
  if (p->err != HYDRA_OK && text) *text = p->err_text;
  return p->err;
}

hydra_status pager_drain(Pager *p, std::string *text) {
  for (int w = 0; w < 2; ++w) {
    Queue &Q = p->queue[w];
    std::unique_lock<std::mutex> l(Q.mu);
    Q.progress.wait(l, [&] { return Q.executed >= Q.submitted; });
  }
  return pager_error(p, text);
}

// Runs on the h2d coordinator.  Chunk by chunk: wait until the ring chunk's previous transfer has left it, fill it
// from the pageable source, hand it to the copy engine.  Returns once every chunk has been ISSUED.
hydra_status pager_h2d(Pager *p, void *dst_dev, const void *src_host, size_t bytes) {
  Ring &r = p->ring[PQ_H2D];
  if (r.n == 0) return HYDRA_E_STATE;  // no staging area
  hipStream_t s = p->ctx->s_h2d;
  if (bytes < (1u << 20)) {
    // small copies (a shard's vectors) share one chunk instead of taking a ring position each
    if (r.small_k < 0 || r.small_off + bytes > r.chunk) {
      r.small_k = (int)(r.next++ % r.n);
      r.small_off = 0;
      if (r.used[r.small_k] && wait_event(p->ctx, r.ev[r.small_k]) != hipSuccess) return HYDRA_E_HIP;
    }
    char *at = r.host + (size_t)r.small_k * r.chunk + r.small_off;
    memcpy(at, src_host, bytes);
    HipGate gate(p->ctx);
    if (hipMemcpyAsync(dst_dev, at, bytes, hipMemcpyHostToDevice, s) != hipSuccess) return HYDRA_E_HIP;
    if (hipEventRecord(r.ev[r.small_k], s) != hipSuccess) return HYDRA_E_HIP;
    r.used[r.small_k] = 1;
    r.small_off += (bytes + 255) & ~(size_t)255;
    return HYDRA_OK;
  }
  for (size_t off = 0; off < bytes; off += r.chunk) {
    const size_t n = bytes - off < r.chunk ? bytes - off : r.chunk;
    const int k = (int)(r.next++ % r.n);
    if (k == r.small_k) r.small_k = -1;  // the ring has come round to the chunk of the small copies
    if (r.used[k] && wait_event(p->ctx, r.ev[k]) != hipSuccess) return HYDRA_E_HIP;
    p->pool[PQ_H2D]->copy(r.host + (size_t)k * r.chunk, (const char *)src_host + off, n);
    HipGate gate(p->ctx);
    if (hipMemcpyAsync((char *)dst_dev + off, r.host + (size_t)k * r.chunk, n, hipMemcpyHostToDevice, s) != hipSuccess)
      return HYDRA_E_HIP;
    if (hipEventRecord(r.ev[k], s) != hipSuccess) return HYDRA_E_HIP;
    r.used[k] = 1;
  }
  return HYDRA_OK;
}

// Runs on the d2h coordinator.  Keeps up to ring-size chunks in flight from the device into the ring and moves each
// into the pageable destination as it lands.  Returns when the data is in dst_host.
// With 'rounded' the bytes are floats and their bf16 roundings are written to rounded[0 .. bytes/4) as well.
hydra_status pager_d2h(Pager *p, void *dst_host, const void *src_dev, size_t bytes, int64_t tokens_per_visit,
                       uint16_t *rounded) {
  Ring &r = p->ring[PQ_D2H];
  if (r.n == 0) return HYDRA_E_STATE;  // no staging area
  hydra_ctx *ctx = p->ctx;
  hipStream_t s = ctx->s_d2h;
  const size_t nchunks = (bytes + r.chunk - 1) / r.chunk;
  size_t issued = 0, drained = 0;
  while (drained < nchunks) {
    while (issued < nchunks && issued - drained < (size_t)r.n) {
      const size_t off = issued * r.chunk;
      const size_t n = bytes - off < r.chunk ? bytes - off : r.chunk;
      const int k = (int)(issued % r.n);  // every chunk of the ring is free when a call starts
      hipError_t e;
      HipGate gate(ctx);
      if (ctx->init.flags & HYDRA_FLAG_D2H_MEMCPY)
        e = hipMemcpyAsync(r.host + (size_t)k * r.chunk, (const char *)src_dev + off, n, hipMemcpyDeviceToHost, s);
      else
        e = launch_copy_to_host(r.mapped + (size_t)k * r.chunk, (const char *)src_dev + off, n, tokens_per_visit,
                                ctx->init.copy_blocks, bytes, s);
      if (e != hipSuccess) return HYDRA_E_HIP;
      if (hipEventRecord(r.ev[k], s) != hipSuccess) return HYDRA_E_HIP;
      ++issued;
    }
    const size_t off = drained * r.chunk;
    const size_t n = bytes - off < r.chunk ? bytes - off : r.chunk;
    const int k = (int)(drained % r.n);
    if (wait_event(ctx, r.ev[k]) != hipSuccess) return HYDRA_E_HIP;
    p->pool[PQ_D2H]->copy((char *)dst_host + off, r.host + (size_t)k * r.chunk, n, rounded ? rounded + off / 4 : nullptr);
    ++drained;
  }
  return HYDRA_OK;
}

}  // namespace hydra
