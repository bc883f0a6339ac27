// Sharded-LRTF scheduler (paper Section 2.4) for one device, and the driver
// that runs its decisions through the swap engine with one task of prefetch
// (double buffering, Section 2.3).
//
// Decision rule: after every shard task, the next task is taken from the model
// whose remaining total time is largest; a shard task is atomic.  Remaining
// time = summed cost of the model's tasks that have not been started; ties go
// to the lowest model index.  The decisions depend only on the cost table, not
// on wall-clock time, so the whole order is computed up front - this also gives
// the buffer manager exact knowledge of future uses.
#include <algorithm>
#include <chrono>

#include "hydra_internal.h"

struct hydra_sched {
  hydra_ctx *ctx = nullptr;
  int n_models = 0;
  std::vector<int> model_id, S, n_mb;
  std::vector<hydra_task> order;  // complete decision sequence; model = index into model_id
  size_t cursor = 0;
  size_t promoted = 0;  // tasks [0, promoted) of the order have had their shard promoted
};

using namespace hydra;

namespace {

struct Chain {
  std::vector<hydra_task> tasks;
  std::vector<int64_t> cost;
};

void build_order(hydra_sched *s, const int64_t *const *task_cost) {
  std::vector<Chain> ch(s->n_models);
  std::vector<int64_t> remaining(s->n_models, 0);
  for (int m = 0; m < s->n_models; ++m) {
    const int ns = s->S[m] + 2;
    for (int mb = 0; mb < s->n_mb[m]; ++mb) {
      for (int sh = 0; sh < ns; ++sh) {
        ch[m].tasks.push_back({m, sh, 0, mb});
        ch[m].cost.push_back(task_cost[m][sh]);
      }
      for (int sh = ns - 1; sh >= 0; --sh) {
        ch[m].tasks.push_back({m, sh, 1, mb});
        ch[m].cost.push_back(task_cost[m][ns + sh]);
      }
    }
    for (int64_t c : ch[m].cost) remaining[m] += c;
  }
  std::vector<size_t> cur(s->n_models, 0);
  for (;;) {
    int best = -1;
    for (int m = 0; m < s->n_models; ++m)
      if (cur[m] < ch[m].tasks.size() && (best < 0 || remaining[m] > remaining[best])) best = m;
    if (best < 0) break;
    s->order.push_back(ch[best].tasks[cur[best]]);
    remaining[best] -= ch[best].cost[cur[best]];
    cur[best]++;
  }
}

// index of the next task at or after 'from' that uses (model, shard); large if none
size_t next_use(const hydra_sched *s, size_t from, int model, int shard) {
  for (size_t i = from; i < s->order.size(); ++i)
    if (s->order[i].model == model && s->order[i].shard == shard) return i;
  return (size_t)-1;
}

// Promote the shard of task j while tasks i .. j-1 have not been enqueued yet.  When no buffer is free, a resident
// shard that none of the tasks i .. j needs is demoted first; returns 1 (not an error) when there is none.
hydra_status promote(hydra_sched *s, size_t j, size_t i) {
  hydra_ctx *ctx = s->ctx;
  const hydra_task &t = s->order[j];
  const int mid = s->model_id[t.model];
  const int what = t.phase == 1 ? (HYDRA_LOAD_PARAMS | HYDRA_LOAD_OPT) : HYDRA_LOAD_PARAMS;
  hydra_status st = ensure_planned(ctx);
  if (st) return st;
  if (!slot_for(ctx, mid, t.shard)) {
    bool has_free = false;
    for (const Slot &sl : ctx->slots) has_free |= sl.model < 0;
    if (!has_free) {
      // Candidates are the buffers not needed again soon.  Among them the one that is free first goes: a buffer
      // whose shard was never written back since it was filled (a forward visit changes nothing) is free at once,
      // otherwise write-backs finish in the order they were enqueued; ties go to the buffer idle longest.  (Taking
      // the buffer idle longest regardless evicted the embedding shard at every step boundary and stalled the
      // promote for the 7 ms its 470 MB write-back still needed.)  If every buffer is needed soon, the one whose
      // next use is furthest away is taken.
      int victim = -1, oldest = -1;
      size_t far = 0;
      uint64_t oldest_use = ~0ull, oldest_wb = ~0ull;
      bool oldest_recent = true;
      const size_t soon = 2 * ctx->slots.size();
      for (size_t q = 0; q < ctx->slots.size(); ++q) {
        const Slot &sl = ctx->slots[q];
        int local = -1;
        for (int m = 0; m < s->n_models; ++m)
          if (s->model_id[m] == sl.model) local = m;
        const size_t nu = local < 0 ? (size_t)-1 : next_use(s, i, local, sl.shard);
        if (nu <= j) continue;  // a task that runs before the prefetched one (or that one itself) works on it
        if (victim < 0 || nu > far) { victim = (int)q; far = nu; }
        const uint64_t wb = sl.dirty ? ~0ull - 1 : sl.wb_seq;  // a write-back not even enqueued yet comes last
        // a buffer that one of the last tasks (one per lane) ran on is free only when that task has finished: its
        // old write-back says nothing (taking it made the promote wait 4 ms per step for a forward visit just enqueued)
        const bool recent = ctx->use_counter - sl.last_use < ctx->lanes.size() && sl.last_use > 0;
        if (nu == (size_t)-1 || nu - i > soon) {
          const bool better = oldest < 0 || (oldest_recent && !recent) ||
                              (oldest_recent == recent && (wb < oldest_wb || (wb == oldest_wb && sl.last_use < oldest_use)));
          if (better) {
            oldest = (int)q;
            oldest_use = sl.last_use;
            oldest_wb = wb;
            oldest_recent = recent;
          }
        }
      }
      if (oldest >= 0) victim = oldest;
      if (victim < 0) return 1;
      const Slot &v = ctx->slots[victim];
      st = hydra_shard_spill(ctx, v.model, v.shard, HYDRA_SPILL_WRITEBACK | HYDRA_SPILL_EVICT);
      if (st) return st;
    }
  }
  return hydra_shard_load_async(ctx, mid, t.shard, what);
}

// adds the host time of a scope to a counter of the context's statistics
struct HostTimer {
  double *acc;
  std::chrono::steady_clock::time_point t0 = std::chrono::steady_clock::now();
  explicit HostTimer(double *a) : acc(a) {}
  ~HostTimer() { *acc += std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count(); }
};

}  // namespace

extern "C" {

hydra_status hydra_sched_create(hydra_ctx *ctx, int32_t n_models, const int32_t *model_ids,
                                const int32_t *n_block_shards, const int32_t *n_minibatches,
                                const int64_t *const *task_cost, hydra_sched **out) {
  if (n_models <= 0 || !n_minibatches || !task_cost || !out) return fail(ctx, HYDRA_E_INVAL, "bad scheduler argument");
  if (ctx && !model_ids) return fail(ctx, HYDRA_E_INVAL, "model ids required with a context");
  if (!ctx && !n_block_shards) return fail(ctx, HYDRA_E_INVAL, "shard counts required without a context");
  hydra_sched *s = new hydra_sched();
  s->ctx = ctx;
  s->n_models = n_models;
  for (int m = 0; m < n_models; ++m) {
    int S;
    if (ctx) {
      if (model_ids[m] < 0 || model_ids[m] >= (int)ctx->models.size()) {
        delete s;
        return fail(ctx, HYDRA_E_INVAL, "unknown model id");
      }
      S = ctx->models[model_ids[m]]->sh.S;
    } else {
      S = n_block_shards[m];
    }
    if (S < 1 || n_minibatches[m] < 0 || !task_cost[m]) {
      delete s;
      return fail(ctx, HYDRA_E_INVAL, "bad per-model scheduler argument");
    }
    for (int i = 0; i < 2 * (S + 2); ++i)
      if (task_cost[m][i] < 0) {
        delete s;
        return fail(ctx, HYDRA_E_INVAL, "negative task cost");
      }
    s->model_id.push_back(ctx ? model_ids[m] : m);
    s->S.push_back(S);
    s->n_mb.push_back(n_minibatches[m]);
  }
  build_order(s, task_cost);
  *out = s;
  return HYDRA_OK;
}

hydra_status hydra_sched_destroy(hydra_sched *s) {
  delete s;
  return HYDRA_OK;
}

hydra_status hydra_sched_next(hydra_sched *s, hydra_task *out) {
  if (!s || !out) return fail(nullptr, HYDRA_E_INVAL, "null argument");
  if (s->cursor >= s->order.size()) return 1;
  *out = s->order[s->cursor++];
  out->model = s->model_id[out->model];
  return HYDRA_OK;
}

hydra_status hydra_sched_run(hydra_sched *s, const int32_t *const *tokens, const int32_t *const *targets,
                             hydra_task *trace, int64_t trace_cap, int64_t *n_executed) {
  if (!s || !s->ctx) return fail(nullptr, HYDRA_E_INVAL, "scheduler has no context");
  hydra_ctx *ctx = s->ctx;
  if (!tokens || !targets) return fail(ctx, HYDRA_E_INVAL, "null batch arrays");
  hydra_status st = ensure_planned(ctx);
  if (st) return st;
  size_t total_shards = 0;
  for (Model *m : ctx->models) total_shards += m->sh.S + 2;
  const bool all_fit = ctx->slots.size() >= total_shards;
  int64_t done = 0;
  // How many tasks ahead shards are promoted for: one (the paper's double buffering) unless the caller asks for
  // more.  Deeper prefetch measured slower with six buffers on the two-model GPT-2-small workload (100.7 ms per
  // step one task ahead, 114 / 112 / 119 ms two / three / six ahead): promotes queue in order on one copy stream, and
  // one that waits for its buffer's write-back holds back the promotes behind it whose buffers are free.
  const size_t depth = ctx->init.prefetch_depth > 0 ? (size_t)ctx->init.prefetch_depth : 1;
  if (s->promoted < s->cursor) s->promoted = s->cursor;
  while (s->cursor < s->order.size()) {
    const size_t i = s->cursor;
    const hydra_task t = s->order[i];
    const int mid = s->model_id[t.model];
    Model *mm = ctx->models[mid];
    // promote this task's shard if that has not happened yet (the previous task's prefetch usually did)
    {
      HostTimer ht(&ctx->stats.host_promote_ms);
      while (s->promoted <= i) {
        st = promote(s, s->promoted, i);
        if (st == 1) return fail(ctx, HYDRA_E_NOSLOT, "no shard buffer can be freed for the next task");
        if (st) return st;
        s->promoted++;
      }
    }
    if (t.phase == 0 && t.shard == 0) {
      HostTimer ht(&ctx->stats.host_batch_ms);
      const int64_t per = mm->sh.Mt;
      if ((st = hydra_set_batch(ctx, mid, tokens[t.model] + t.minibatch * per, targets[t.model] + t.minibatch * per)))
        return st;
    }
    if (t.phase == 0) {
      HostTimer ht(&ctx->stats.host_task_ms);
      if ((st = hydra_shard_forward(ctx, mid, t.shard))) return st;
    } else {
      {
        HostTimer ht(&ctx->stats.host_task_ms);
        if ((st = hydra_shard_backward(ctx, mid, t.shard))) return st;
        if ((st = hydra_shard_adam_step(ctx, mid, t.shard))) return st;
      }
      // when shards do not all fit, start the write-back right away so that it
      // overlaps the following tasks instead of delaying the next promote
      if (!all_fit) {
        HostTimer ht(&ctx->stats.host_writeback_ms);
        if ((st = hydra_shard_spill(ctx, mid, t.shard, HYDRA_SPILL_WRITEBACK))) return st;
      }
    }
    if (trace && done < trace_cap) {
      trace[done] = t;
      trace[done].model = mid;
    }
    ++done;
    s->cursor++;
    // Prefetch the shards of the tasks after this one while it runs (double buffering, paper Section 2.3; deeper
    // where the caller asks for it).  After the task has been enqueued, not before: a promote call returns only
    // when what the promote depends on has finished, and the device should be computing meanwhile.
    {
      HostTimer ht(&ctx->stats.host_promote_ms);
      while (s->promoted < s->order.size() && s->promoted <= i + depth) {
        st = promote(s, s->promoted, i + 1);
        if (st == 1) break;  // every buffer holds a shard that a task before that one needs
        if (st) return st;
        s->promoted++;
      }
    }
  }
  if (n_executed) *n_executed = done;
  return HYDRA_OK;
}

}  // extern "C"
