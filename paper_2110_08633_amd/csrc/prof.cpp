// Optional per-kernel timing with HIP events on the stream a kernel is
// launched on (enabled by HYDRA_FLAG_TIMING).  Each launch is bracketed by two
// events; after a synchronisation the elapsed times are aggregated per kernel
// name together with the algorithmic flops / bytes of the launches.
#include <map>

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
  std::vector<ProfRec> recs;
  std::vector<hipEvent_t> pool;
  std::map<std::string, ProfAgg> agg;
  std::vector<std::string> order;
};

static Profiler *g_prof = nullptr;

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
  if (!p) return;
  ProfRec r{name, get_event(p), get_event(p), flops, bytes};
  if (!r.e0 || !r.e1) return;
  (void)hipEventRecord(r.e0, s);
  p->recs.push_back(r);
  idx_ = (long)p->recs.size() - 1;
}

ProfScope::~ProfScope() {
  Profiler *p = g_prof;
  if (!p || idx_ < 0) return;
  (void)hipEventRecord(p->recs[idx_].e1, stream_);
}

// caller has synchronised the streams
void prof_collect(Profiler *p) {
  for (ProfRec &r : p->recs) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.e0, r.e1) == hipSuccess) {
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
  prof_collect(p);
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

}  // namespace hydra

using namespace hydra;

extern "C" {

hydra_status hydra_kernel_stats(hydra_ctx *ctx, int32_t index, char name[64], uint64_t *launches, double *total_ms,
                                double *flops, double *bytes) {
  if (!ctx || !name || !launches || !total_ms || !flops || !bytes) return fail(ctx, HYDRA_E_INVAL, "null argument");
  if (!ctx->prof) return fail(ctx, HYDRA_E_STATE, "context was not created with HYDRA_FLAG_TIMING");
  hydra_status st = hydra_sync(ctx);
  if (st) return st;
  prof_collect(ctx->prof);
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
