// Optional per-kernel timing with HIP events on the stream a kernel is
// launched on (enabled by HYDRA_FLAG_TIMING).  Each launch is bracketed by two
// events; after a synchronisation the elapsed times are aggregated per kernel
// name together with the algorithmic flops / bytes of the launches.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>

#include "hydra_internal.h"

namespace hydra {

struct ProfRec {
  const char *name;
  hipEvent_t e0, e1;
  double flops, bytes;
};

struct ProfAgg {
  uint64_t launches = 0;
  double ms = 0, flops = 0, bytes = 0;
};

struct Profiler {
  std::mutex mu;  // launches come from the calling thread and, with a staging tier, from its coordinator threads
  std::vector<ProfRec> recs;
  std::vector<std::pair<double, double>> ivals;  // launch intervals (ms after the overlap trace's base event)
  std::vector<hipEvent_t> pool;
  std::map<std::string, ProfAgg> agg;
  std::vector<std::string> order;
};

static Profiler *g_prof = nullptr;
static thread_local int g_prof_quiet = 0;

ProfSuppress::ProfSuppress() { ++g_prof_quiet; }
ProfSuppress::~ProfSuppress() { --g_prof_quiet; }

Profiler *prof_create() { return new Profiler(); }
void prof_destroy(Profiler *p) {
  if (!p) return;
  if (g_prof == p) g_prof = nullptr;
  for (ProfRec &r : p->recs) {
    (void)hipEventDestroy(r.e0);
    (void)hipEventDestroy(r.e1);
  }
  for (hipEvent_t e : p->pool) (void)hipEventDestroy(e);
  delete p;
}
void prof_activate(Profiler *p) { g_prof = p; }

static hipEvent_t get_event(Profiler *p) {
  if (!p->pool.empty()) {
    hipEvent_t e = p->pool.back();
    p->pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

ProfScope::ProfScope(const char *name, hipStream_t s, double flops, double bytes) : stream_(s), idx_(-1) {
  Profiler *p = g_prof;
  if (!p || g_prof_quiet) return;
  std::lock_guard<std::mutex> lock(p->mu);
  ProfRec r{name, get_event(p), get_event(p), flops, bytes};
  if (!r.e0 || !r.e1) return;
  (void)hipEventRecord(r.e0, s);
  p->recs.push_back(r);
  idx_ = (long)p->recs.size() - 1;
}

ProfScope::~ProfScope() {
  Profiler *p = g_prof;
  if (!p || idx_ < 0) return;
  std::lock_guard<std::mutex> lock(p->mu);
  (void)hipEventRecord(p->recs[idx_].e1, stream_);
}

// caller has synchronised the streams.  base (may be null): an event recorded before all of these launches; the
// launches' intervals relative to it are kept for the overlap trace.
void prof_collect(Profiler *p, hipEvent_t base) {
  std::lock_guard<std::mutex> lock(p->mu);
  for (ProfRec &r : p->recs) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.e0, r.e1) == hipSuccess) {
      float a = 0.f;
      // (the write-back's copy kernel is a transfer, not compute)
      if (base && strcmp(r.name, "copy_to_host") != 0 && hipEventElapsedTime(&a, base, r.e0) == hipSuccess && a >= 0.f)
        p->ivals.push_back({a, a + ms});
      auto it = p->agg.find(r.name);
      if (it == p->agg.end()) {
        p->order.push_back(r.name);
        it = p->agg.emplace(r.name, ProfAgg()).first;
      }
      it->second.launches++;
      it->second.ms += ms;
      it->second.flops += r.flops;
      it->second.bytes += r.bytes;
    }
    p->pool.push_back(r.e0);
    p->pool.push_back(r.e1);
  }
  p->recs.clear();
}

void prof_reset(Profiler *p) {
  prof_collect(p, nullptr);
  p->ivals.clear();
  p->agg.clear();
  p->order.clear();
}

int prof_count(Profiler *p) { return (int)p->order.size(); }
bool prof_get(Profiler *p, int i, std::string *name, uint64_t *launches, double *ms, double *flops, double *bytes) {
  if (i < 0 || i >= (int)p->order.size()) return false;
  const ProfAgg &a = p->agg[p->order[i]];
  *name = p->order[i];
  *launches = a.launches;
  *ms = a.ms;
  *flops = a.flops;
  *bytes = a.bytes;
  return true;
}

// ---------------------------------------------------------------------------
// Swap / compute overlap (HYDRA_FLAG_OVERLAP): an event pair around every
// promote, write-back and shard task, each on the stream the operation runs
// on; the host turns the timestamps into interval unions after a
// synchronisation.
// ---------------------------------------------------------------------------
struct TraceRec {
  int kind, tag;
  hipEvent_t e0, e1;
  uint64_t bytes;
  bool closed;
};

struct Tracer {
  std::mutex mu;  // intervals are opened by the calling thread and by the staging tier's coordinator threads
  std::vector<TraceRec> recs;
  std::vector<hipEvent_t> pool;
  hipEvent_t base = nullptr;
  bool base_recorded = false;
};

Tracer *trace_create() { return new Tracer(); }

void trace_destroy(Tracer *t) {
  if (!t) return;
  for (TraceRec &r : t->recs) {
    (void)hipEventDestroy(r.e0);
    (void)hipEventDestroy(r.e1);
  }
  for (hipEvent_t e : t->pool) (void)hipEventDestroy(e);
  if (t->base) (void)hipEventDestroy(t->base);
  delete t;
}

static hipEvent_t trace_event(Tracer *t) {
  if (!t->pool.empty()) {
    hipEvent_t e = t->pool.back();
    t->pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

int trace_begin(hydra_ctx *ctx, int kind, hipStream_t s, int tag) {
  Tracer *t = ctx->tracer;
  if (!t) return -1;
  std::lock_guard<std::mutex> lock(t->mu);
  if (!t->base_recorded) {
    if (!t->base && hipEventCreate(&t->base) != hipSuccess) return -1;
    if (hipEventRecord(t->base, s) != hipSuccess) return -1;
    t->base_recorded = true;
  }
  TraceRec r{kind, tag, trace_event(t), trace_event(t), 0, false};
  if (!r.e0 || !r.e1) return -1;
  // The start event follows an empty kernel: a kernel is held back by the waits enqueued before it, so the interval
  // opens when the stream has actually reached the operation (an event recorded directly after a wait for another
  // stream's event was seen to carry a time stamp from before that wait was satisfied).
  (void)launch_stream_marker(s);
  (void)hipEventRecord(r.e0, s);
  t->recs.push_back(r);
  return (int)t->recs.size() - 1;
}

void trace_end(hydra_ctx *ctx, int idx, hipStream_t s, uint64_t bytes) {
  Tracer *t = ctx->tracer;
  if (!t || idx < 0) return;
  std::lock_guard<std::mutex> lock(t->mu);
  if (idx >= (int)t->recs.size()) return;
  (void)hipEventRecord(t->recs[idx].e1, s);
  t->recs[idx].bytes = bytes;
  t->recs[idx].closed = true;
}

typedef std::vector<std::pair<double, double>> Intervals;

// sorted, disjoint union of a set of intervals
static Intervals merged(Intervals v) {
  std::sort(v.begin(), v.end());
  Intervals out;
  for (const auto &iv : v) {
    if (!out.empty() && iv.first <= out.back().second) out.back().second = std::max(out.back().second, iv.second);
    else out.push_back(iv);
  }
  return out;
}
static double length(const Intervals &v) {
  double s = 0;
  for (const auto &iv : v) s += iv.second - iv.first;
  return s;
}
// length of the intersection of two sorted disjoint unions
static double common(const Intervals &a, const Intervals &b) {
  double s = 0;
  size_t i = 0, j = 0;
  while (i < a.size() && j < b.size()) {
    const double lo = std::max(a[i].first, b[j].first), hi = std::min(a[i].second, b[j].second);
    if (hi > lo) s += hi - lo;
    if (a[i].second < b[j].second) ++i;
    else ++j;
  }
  return s;
}

// caller has synchronised the streams.  dump (may be null): one line per interval (kind, model, shard, start ms, end
// ms, bytes).  prof (may be null): per-kernel timing of the same context, whose launch intervals give the
// kernel-level figures.
static void trace_collect(Tracer *t, Profiler *prof, hydra_overlap *out, FILE *dump) {
  memset(out, 0, sizeof *out);
  Intervals by_kind[3];
  double lo = 1e300, hi = -1e300;
  for (TraceRec &r : t->recs) {
    float a = 0.f, b = 0.f;
    if (r.closed && hipEventElapsedTime(&a, t->base, r.e0) == hipSuccess &&
        hipEventElapsedTime(&b, t->base, r.e1) == hipSuccess && b >= a) {
      if (dump)
        fprintf(dump, "%s %d %d %.4f %.4f %llu\n", r.kind == TRACE_COMPUTE ? "compute" : r.kind == TRACE_H2D ? "h2d" : "d2h",
                r.tag >> 16, r.tag & 0xffff, a, b, (unsigned long long)r.bytes);
      by_kind[r.kind].push_back({a, b});
      lo = std::min(lo, (double)a);
      hi = std::max(hi, (double)b);
      if (r.kind == TRACE_H2D) out->bytes_h2d += r.bytes;
      if (r.kind == TRACE_D2H) out->bytes_d2h += r.bytes;
      out->n_intervals++;
    }
  }
  (void)hipGetLastError();
  if (!out->n_intervals) return;
  const Intervals comp = merged(by_kind[TRACE_COMPUTE]), h2d = merged(by_kind[TRACE_H2D]),
                  d2h = merged(by_kind[TRACE_D2H]);
  Intervals both = h2d;
  both.insert(both.end(), d2h.begin(), d2h.end());
  const Intervals xfer = merged(both);
  out->wall_ms = hi - lo;
  out->compute_ms = length(comp);
  out->h2d_ms = length(h2d);
  out->d2h_ms = length(d2h);
  out->transfer_ms = length(xfer);
  out->hidden_ms = common(xfer, comp);
  if (prof) {
    prof_collect(prof, t->base_recorded ? t->base : nullptr);
    (void)hipGetLastError();
    const Intervals kern = merged(prof->ivals);
    out->kernel_ms = length(kern);
    out->hidden_kernel_ms = common(xfer, kern);
    if (dump)
      for (const auto &iv : prof->ivals) fprintf(dump, "kernel -1 -1 %.4f %.4f 0\n", iv.first, iv.second);
  }
}

static void trace_reset(Tracer *t, Profiler *prof) {
  if (prof) prof->ivals.clear();
  for (TraceRec &r : t->recs) {
    t->pool.push_back(r.e0);
    t->pool.push_back(r.e1);
  }
  t->recs.clear();
  t->base_recorded = false;
}

}  // namespace hydra

using namespace hydra;

extern "C" {

hydra_status hydra_overlap_stats(hydra_ctx *ctx, hydra_overlap *out) {
  if (!ctx || !out) return fail(ctx, HYDRA_E_INVAL, "null argument");
  if (!ctx->tracer) return fail(ctx, HYDRA_E_STATE, "context was not created with HYDRA_FLAG_OVERLAP");
  hydra_status st = hydra_sync(ctx);
  if (st) return st;
  trace_collect(ctx->tracer, ctx->prof, out, nullptr);
  return HYDRA_OK;
}

hydra_status hydra_overlap_dump(hydra_ctx *ctx, const char *path) {
  if (!ctx || !path) return fail(ctx, HYDRA_E_INVAL, "null argument");
  if (!ctx->tracer) return fail(ctx, HYDRA_E_STATE, "context was not created with HYDRA_FLAG_OVERLAP");
  hydra_status st = hydra_sync(ctx);
  if (st) return st;
  FILE *f = fopen(path, "w");
  if (!f) return fail(ctx, HYDRA_E_INVAL, std::string("cannot open ") + path);
  hydra_overlap o;
  trace_collect(ctx->tracer, ctx->prof, &o, f);
  fclose(f);
  return HYDRA_OK;
}

hydra_status hydra_overlap_reset(hydra_ctx *ctx) {
  if (!ctx) return fail(ctx, HYDRA_E_INVAL, "null argument");
  if (!ctx->tracer) return fail(ctx, HYDRA_E_STATE, "context was not created with HYDRA_FLAG_OVERLAP");
  hydra_status st = hydra_sync(ctx);
  if (st) return st;
  trace_reset(ctx->tracer, ctx->prof);
  return HYDRA_OK;
}

hydra_status hydra_kernel_stats(hydra_ctx *ctx, int32_t index, char name[64], uint64_t *launches, double *total_ms,
                                double *flops, double *bytes) {
  if (!ctx || !name || !launches || !total_ms || !flops || !bytes) return fail(ctx, HYDRA_E_INVAL, "null argument");
  if (!ctx->prof) return fail(ctx, HYDRA_E_STATE, "context was not created with HYDRA_FLAG_TIMING");
  hydra_status st = hydra_sync(ctx);
  if (st) return st;
  prof_collect(ctx->prof, ctx->tracer && ctx->tracer->base_recorded ? ctx->tracer->base : nullptr);
  std::string n;
  if (!prof_get(ctx->prof, index, &n, launches, total_ms, flops, bytes)) return 1;
  snprintf(name, 64, "%s", n.c_str());
  return HYDRA_OK;
}

hydra_status hydra_kernel_stats_reset(hydra_ctx *ctx) {
  if (!ctx) return fail(ctx, HYDRA_E_INVAL, "null argument");
  if (!ctx->prof) return fail(ctx, HYDRA_E_STATE, "context was not created with HYDRA_FLAG_TIMING");
  hydra_status st = hydra_sync(ctx);
  if (st) return st;
  prof_reset(ctx->prof);
  return HYDRA_OK;
}

}  // extern "C"
