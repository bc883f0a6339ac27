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
#include <atomic>
#include <condition_variable>
#include <cstring>
#include <deque>
#include <functional>
#include <mutex>
#include <thread>

#include "hydra_internal.h"

namespace hydra {

namespace {

// n bytes copied by the calling thread and a few helpers, each a contiguous part
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
  void copy(void *dst, const void *src, size_t n) {
    const size_t parts = th_.size() + 1;
    if (n < (1u << 20) || parts == 1) {
      memcpy(dst, src, n);
      return;
    }
    const size_t per = (n / parts + 4095) & ~(size_t)4095;
    {
      std::lock_guard<std::mutex> l(mu_);
      dst_ = (char *)dst; src_ = (const char *)src; n_ = n; per_ = per;
      pending_ = (int)th_.size();
      ++gen_;
    }
    cv_.notify_all();
    memcpy(dst, src, per < n ? per : n);  // part 0
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
      l.unlock();
      if (lo < hi) memcpy(d + lo, s + lo, hi - lo);
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
  hipStream_t s = p->ctx->s_h2d;
  for (size_t off = 0; off < bytes; off += r.chunk) {
    const size_t n = bytes - off < r.chunk ? bytes - off : r.chunk;
    const int k = (int)(r.next++ % r.n);
    if (r.used[k] && hipEventSynchronize(r.ev[k]) != hipSuccess) return HYDRA_E_HIP;
    p->pool[PQ_H2D]->copy(r.host + (size_t)k * r.chunk, (const char *)src_host + off, n);
    if (hipMemcpyAsync((char *)dst_dev + off, r.host + (size_t)k * r.chunk, n, hipMemcpyHostToDevice, s) != hipSuccess)
      return HYDRA_E_HIP;
    if (hipEventRecord(r.ev[k], s) != hipSuccess) return HYDRA_E_HIP;
    r.used[k] = 1;
  }
  return HYDRA_OK;
}

// Runs on the d2h coordinator.  Keeps up to ring-size chunks in flight from the device into the ring and moves each
// into the pageable destination as it lands.  Returns when the data is in dst_host.
hydra_status pager_d2h(Pager *p, void *dst_host, const void *src_dev, size_t bytes, int64_t tokens_per_visit) {
  Ring &r = p->ring[PQ_D2H];
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
    if (hipEventSynchronize(r.ev[k]) != hipSuccess) return HYDRA_E_HIP;
    p->pool[PQ_D2H]->copy((char *)dst_host + off, r.host + (size_t)k * r.chunk, n);
    ++drained;
  }
  return HYDRA_OK;
}

}  // namespace hydra
