// Context, shard buffers (slots) and the swap engine: promote / demote of
// shard state between pinned host arrays and device buffers on dedicated copy
// streams, ordered against the compute stream by events only (paper Section
// 2.3: spilling with double buffering).
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "hydra_internal.h"

namespace hydra {

const char *global_error();

hydra_status fail(hydra_ctx *ctx, hydra_status code, const std::string &msg) {
  if (ctx) ctx->err = msg;
  else set_global_error(msg);
  return code;
}

hydra_status hipfail(hydra_ctx *ctx, hipError_t e, const char *what) {
  std::string m = std::string("HIP error '") + hipGetErrorString(e) + "' at " + what;
  return fail(ctx, HYDRA_E_HIP, m);
}

static inline uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

static char *arena_take(hydra_ctx *ctx, uint64_t bytes) {
  const uint64_t off = align_up(ctx->arena_used, 256);
  if (off + bytes > ctx->arena_bytes) return nullptr;
  ctx->arena_used = off + bytes;
  return ctx->arena + off;
}

Slot *slot_for(hydra_ctx *ctx, int model, int shard) {
  const int i = ctx->models[model]->slot_of[shard];
  return i < 0 ? nullptr : &ctx->slots[i];
}

hydra_status copy_d2h(hydra_ctx *ctx, void *host_dst, void *host_dst_mapped, const void *src, size_t bytes,
                      int64_t tokens_per_visit) {
  if (ctx->dry) return HYDRA_OK;
  if (ctx->init.flags & HYDRA_FLAG_D2H_MEMCPY)
    HYDRA_HIP(ctx, hipMemcpyAsync(host_dst, src, bytes, hipMemcpyDeviceToHost, ctx->s_d2h));
  else
    HYDRA_HIP(ctx, launch_copy_to_host(host_dst_mapped, src, bytes, tokens_per_visit, ctx->init.copy_blocks, bytes, ctx->s_d2h));
  return HYDRA_OK;
}

// What one promote or one write-back puts on its copy stream: waits for events other streams recorded, copies, and
// events to record behind them.  Without a staging tier the calling thread issues it at once; with one it is a job
// of that direction's coordinator thread (pager.cpp), which is why nothing in here may touch the context's
// bookkeeping or its error text.
struct CopyPlan {
  struct Seg {
    void *dst;
    const void *src;
    void *dst_mapped;  // write-backs into page-locked memory: the destination as the device sees it
    size_t bytes;
    int kind;          // SEG_*
    uint16_t *rounded = nullptr;  // staged write-backs of the master: where the host threads leave its bf16 rounding
  };
  enum { SEG_PINNED = 0, SEG_PAGEABLE = 1, SEG_DEVICE = 2 };
  std::vector<hipEvent_t> waits;
  std::vector<uint64_t> d2h_tickets;  // staging tier: write-back jobs that must have finished first
  std::vector<Seg> segs;
  std::vector<hipEvent_t> records;
  int trace_tag = 0;
  uint64_t trace_bytes = 0;
  int64_t tokens_per_visit = 0;
  bool poison = false;                // write-backs: fill the whole buffer with NaN patterns afterwards
  void *poison_base = nullptr;
  int64_t poison_words = 0;
};

#define PLAN_HIP(call)                            \
  do {                                            \
    if ((call) != hipSuccess) return HYDRA_E_HIP; \
  } while (0)

// Both functions run on the coordinator thread of their direction.  Calls into the HIP runtime are made inside a
// HipGate scope and events are waited for with wait_event (see hydra_ctx::hip_gate).
static hydra_status run_h2d_plan(hydra_ctx *ctx, const CopyPlan &p) {
  hipStream_t s = ctx->s_h2d;
  for (uint64_t t : p.d2h_tickets) pager_wait(ctx->pager, PQ_D2H, t);
  // The thread waits for what the promote depends on (the write-back that frees its buffer, the one that brought
  // the shard's state to the host) and only then hands the copies to the stream.  Enqueued behind stream waits
  // instead, the same copies ran slower: four GPT-2-medium models 14.1 k -> 16.2-17.5 k tokens/s with the waits on
  // the host, two GPT-2-small models 35.8 k -> 41.5 k (the link was then used to 0.93-1.0 of its measured two-way
  // rate instead of 0.80-0.85).  Every event in the list was recorded before the plan was made, by work that
  // depends on nothing enqueued later, so the wait ends.
  for (hipEvent_t e : p.waits) PLAN_HIP(wait_event(ctx, e));
  int tr = -1;
  if (p.trace_bytes) {
    HipGate gate(ctx);
    tr = trace_begin(ctx, TRACE_H2D, s, p.trace_tag);
  }
  for (const CopyPlan::Seg &g : p.segs) {
    if (g.kind == CopyPlan::SEG_PAGEABLE) {
      const hydra_status st = pager_h2d(ctx->pager, g.dst, g.src, g.bytes);
      if (st) return st;
    } else {
      // SDMA (hipMemcpyAsync): the copy kernel reading page-locked memory through its device-side mapping reaches the
      // same link rate but slows the compute kernels it shares CUs with and the write-backs (measured: 147 against
      // 123 ms per step of the two-model GPT-2-small workload)
      HipGate gate(ctx);
      PLAN_HIP(hipMemcpyAsync(g.dst, g.src, g.bytes,
                              g.kind == CopyPlan::SEG_DEVICE ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, s));
    }
  }
  HipGate gate(ctx);
  trace_end(ctx, tr, s, p.trace_bytes);
  for (hipEvent_t e : p.records) PLAN_HIP(hipEventRecord(e, s));
  return HYDRA_OK;
}

static hydra_status run_d2h_plan(hydra_ctx *ctx, const CopyPlan &p) {
  hipStream_t s = ctx->s_d2h;
  // as for promotes: the thread waits for the task that last used the buffer, then issues the copies
  for (hipEvent_t e : p.waits) PLAN_HIP(wait_event(ctx, e));
  int tr = -1;
  if (p.trace_bytes) {
    HipGate gate(ctx);
    tr = trace_begin(ctx, TRACE_D2H, s, p.trace_tag);
  }
  for (const CopyPlan::Seg &g : p.segs) {
    if (g.kind == CopyPlan::SEG_PAGEABLE) {
      const hydra_status st = pager_d2h(ctx->pager, g.dst, g.src, g.bytes, p.tokens_per_visit, g.rounded);
      if (st) return st;
    } else if (!(ctx->init.flags & HYDRA_FLAG_D2H_KERNEL)) {
      // Page-locked state: hipMemcpyAsync (which this runtime executes as a copy kernel of its own, not on a copy
      // engine).  Issued like this - by a thread that has waited for the task, so that the copy can start at once -
      // it carries 49-50 GB/s next to the promotes and hardly touches the compute kernels, where the library's
      // copy kernel carries 41-47 and slows every kernel on the device (two GPT-2-small models
      // 42.7 k -> 43.8 k tokens/s, four GPT-2-medium models 17.4 k -> 18.6 k, eight micro-batches per visit 287 k ->
      // 333 k).  Enqueued behind a stream wait the same copies reached 25-35 GB/s.  State behind the staging area
      // stays with the copy kernel: through the ring's 64 MiB chunks the runtime's copy was faster on some runs and
      // slower on others (two 6 B models: 507 / 534 / 470 tokens/s against 526-528).
      HipGate gate(ctx);
      PLAN_HIP(hipMemcpyAsync(g.dst, g.src, g.bytes, hipMemcpyDeviceToHost, s));
    } else {
      HipGate gate(ctx);
      PLAN_HIP(launch_copy_to_host(g.dst_mapped, g.src, g.bytes, p.tokens_per_visit, ctx->init.copy_blocks, g.bytes, s));
    }
  }
  HipGate gate(ctx);
  trace_end(ctx, tr, s, p.trace_bytes);
  if (p.poison) PLAN_HIP(launch_fill_u32((uint32_t *)p.poison_base, 0x7fc07fc0u, p.poison_words, s));
  for (hipEvent_t e : p.records) PLAN_HIP(hipEventRecord(e, s));
  return HYDRA_OK;
}

// Issues a plan: at once, or as a job of the staging tier's coordinator for that direction (ticket returned).
static hydra_status issue_plan(hydra_ctx *ctx, int which, const CopyPlan &p, uint64_t *ticket) {
  *ticket = 0;
  if (ctx->dry) return HYDRA_OK;
  if (!ctx->pager) {
    const hydra_status st = which == PQ_H2D ? run_h2d_plan(ctx, p) : run_d2h_plan(ctx, p);
    if (st) return fail(ctx, st, which == PQ_H2D ? "a HIP call of a promote failed" : "a HIP call of a write-back failed");
    return HYDRA_OK;
  }
  *ticket = pager_submit(ctx->pager, which,
                         [ctx, which, p]() { return which == PQ_H2D ? run_h2d_plan(ctx, p) : run_d2h_plan(ctx, p); });
  return HYDRA_OK;
}

// an error of the staging tier's threads surfaces at the next call that touches the swap engine
static hydra_status pager_check(hydra_ctx *ctx) {
  if (!ctx->pager) return HYDRA_OK;
  std::string text;
  const hydra_status st = pager_error(ctx->pager, &text);
  return st ? fail(ctx, st, text) : HYDRA_OK;
}

// waits until the staging tier's coordinators have nothing left to issue (no-op without one)
hydra_status drain_copies(hydra_ctx *ctx) {
  if (!ctx->pager) return HYDRA_OK;
  std::string text;
  const hydra_status st = pager_drain(ctx->pager, &text);
  return st ? fail(ctx, st, text) : HYDRA_OK;
}

// device-side address of caller memory that must be page-locked and mapped
// (state: one of master / adam_m / adam_v, which the library's copy kernel writes only with HYDRA_FLAG_D2H_KERNEL;
// checkpoints go through it unless HYDRA_FLAG_D2H_MEMCPY is set)
static hydra_status mapped_pointer(hydra_ctx *ctx, const void *host, const char *what, float **out, bool state = false) {
  *out = (float *)host;
  // the device-side mapping is what the library's copy kernel stores through; hipMemcpyAsync takes the host address
  const bool kernel_writes_it = state ? (ctx->init.flags & HYDRA_FLAG_D2H_KERNEL) != 0 : !(ctx->init.flags & HYDRA_FLAG_D2H_MEMCPY);
  if (ctx->dry || !host || !kernel_writes_it) return HYDRA_OK;
  hipPointerAttribute_t at;
  hipError_t e = hipPointerGetAttributes(&at, host);
  if (e != hipSuccess || at.type != hipMemoryTypeHost || !at.devicePointer) {
    (void)hipGetLastError();
    return fail(ctx, HYDRA_E_INVAL, std::string(what) + " is not page-locked host memory");
  }
  if (((uintptr_t)at.devicePointer) & 15) return fail(ctx, HYDRA_E_INVAL, std::string(what) + " must be 16-byte aligned");
  *out = (float *)at.devicePointer;
  return HYDRA_OK;
}

static bool page_locked(const void *host) {
  hipPointerAttribute_t at;
  const bool yes = hipPointerGetAttributes(&at, host) == hipSuccess && at.type == hipMemoryTypeHost;
  if (!yes) (void)hipGetLastError();
  return yes;
}

static hydra_status make_event(hydra_ctx *ctx, hipEvent_t *ev) {
  if (ctx->dry) return HYDRA_OK;
  HYDRA_HIP(ctx, hipEventCreateWithFlags(ev, hipEventDisableTiming));
  return HYDRA_OK;
}

// Carve the rest of the arena into the shared workspace and the shard buffers.
hydra_status ensure_planned(hydra_ctx *ctx) {
  if (ctx->planned) return HYDRA_OK;
  if (ctx->models.empty()) return fail(ctx, HYDRA_E_STATE, "no model registered");
  uint64_t ws = 0, max_shard = 0, total_shards = 0;
  for (Model *m : ctx->models) {
    const uint64_t need = workspace_need(m->sh, m->dtype);
    if (need > ws) ws = need;
    if ((uint64_t)m->sh.max_shard > max_shard) max_shard = m->sh.max_shard;
    total_shards += m->sh.S + 2;
  }
  ctx->stats.model_state_bytes = ctx->arena_used;
  ctx->ws_bytes = align_up(ws, 256);
  for (hydra_ctx::Lane &ln : ctx->lanes) {
    ln.ws = arena_take(ctx, ctx->ws_bytes);
    if (!ln.ws) return fail(ctx, HYDRA_E_NOMEM, "device arena too small for the workspace");
  }
  // a slot: fp32 master, m, v, grad and two bf16 working copies (as stored / matrices transposed) of the largest shard
  ctx->slot_elems = align_up(max_shard, 64);
  ctx->slot_bytes = align_up(ctx->slot_elems * 20, 256);
  const uint64_t base = align_up(ctx->arena_used, 256);
  uint64_t room = ctx->arena_bytes > base ? ctx->arena_bytes - base : 0;
  if (ctx->init.shard_buffer_cap_bytes && ctx->init.shard_buffer_cap_bytes < room)
    room = ctx->init.shard_buffer_cap_bytes;
  uint64_t n = room / ctx->slot_bytes;
  if (ctx->init.max_slots > 0 && n > (uint64_t)ctx->init.max_slots) n = ctx->init.max_slots;
  if (n > total_shards) n = total_shards;
  if (n < 1) return fail(ctx, HYDRA_E_NOMEM, "no room for a single shard buffer (arena or cap too small)");
  ctx->slots.resize(n);
  for (uint64_t i = 0; i < n; ++i) {
    Slot &s = ctx->slots[i];
    s.base = arena_take(ctx, ctx->slot_bytes);
    if (!s.base) return fail(ctx, HYDRA_E_NOMEM, "device arena too small for the shard buffers");
    s.w = (float *)s.base;
    s.m = s.w + ctx->slot_elems;
    s.v = s.m + ctx->slot_elems;
    s.g = s.v + ctx->slot_elems;
    s.wb = (bf16_t *)(s.g + ctx->slot_elems);
    s.wbt = s.wb + ctx->slot_elems;
    hydra_status st;
    if ((st = make_event(ctx, &s.ev_loaded)) || (st = make_event(ctx, &s.ev_compute)) ||
        (st = make_event(ctx, &s.ev_spilled)))
      return st;
  }
  ctx->stats.n_slots = (int32_t)n;
  ctx->stats.slot_bytes = ctx->slot_bytes;
  ctx->stats.workspace_bytes = ctx->ws_bytes * ctx->lanes.size();
  ctx->planned = true;
  return HYDRA_OK;
}

static void destroy_model_events(Model *m) {
  for (int i = 0; i < 2; ++i) {
    if (m->ev_stage[i]) (void)hipEventDestroy(m->ev_stage[i]);
    if (m->ev_ckpt_d2h[i]) (void)hipEventDestroy(m->ev_ckpt_d2h[i]);
    if (m->ev_ckpt_h2d[i]) (void)hipEventDestroy(m->ev_ckpt_h2d[i]);
  }
  if (m->ev_last_compute) (void)hipEventDestroy(m->ev_last_compute);
  for (hipEvent_t e : m->ev_wb)
    if (e) (void)hipEventDestroy(e);
}

static hydra_status check_model(hydra_ctx *ctx, int model, int shard) {
  if (!ctx) return fail(nullptr, HYDRA_E_INVAL, "null context");
  if (model < 0 || model >= (int)ctx->models.size()) return fail(ctx, HYDRA_E_INVAL, "model index out of range");
  if (shard < 0 || shard >= ctx->models[model]->sh.S + 2) return fail(ctx, HYDRA_E_INVAL, "shard index out of range");
  return HYDRA_OK;
}

}  // namespace hydra

using namespace hydra;

extern "C" {

hydra_status hydra_init(const hydra_init_desc *desc, hydra_ctx **out) {
  if (!desc || !out) return fail(nullptr, HYDRA_E_INVAL, "null argument");
  if (!desc->dev_arena || desc->dev_arena_bytes == 0) return fail(nullptr, HYDRA_E_INVAL, "empty device arena");
  if (((uintptr_t)desc->dev_arena) & 255) return fail(nullptr, HYDRA_E_INVAL, "device arena must be 256-byte aligned");
  hydra_ctx *ctx = new hydra_ctx();
  ctx->init = *desc;
  ctx->dry = (desc->flags & HYDRA_FLAG_DRY_RUN) != 0;
  const int n_lanes = desc->compute_lanes > 0 ? desc->compute_lanes : 1;
  if (n_lanes > HYDRA_MAX_LANES) {
    delete ctx;
    return fail(nullptr, HYDRA_E_INVAL, "at most HYDRA_MAX_LANES compute lanes");
  }
  ctx->lanes.resize(n_lanes);
  ctx->lanes[0].stream = (hipStream_t)desc->compute_stream;
  ctx->s_h2d = (hipStream_t)desc->h2d_stream;
  ctx->s_d2h = (hipStream_t)desc->d2h_stream;
  ctx->arena = (char *)desc->dev_arena;
  ctx->arena_bytes = desc->dev_arena_bytes;
  memset(&ctx->stats, 0, sizeof ctx->stats);
  if (!ctx->dry) {
    int n = 0;
    hipError_t e = hipGetDeviceCount(&n);
    if (e != hipSuccess || n < 1) {
      delete ctx;
      return fail(nullptr, HYDRA_E_HIP, "no HIP device available");
    }
  }
  if (!ctx->dry) {  // set-up of the entry point that may not allocate later on: resolve this GPU's scratch array now
    float *unused = nullptr;
    const hydra_status ss = static_scratch(&unused);
    if (ss) {
      delete ctx;
      return ss;
    }
  }
  for (int i = 1; i < n_lanes && !ctx->dry; ++i) {
    hipStream_t ls = (hipStream_t)desc->lane_streams[i - 1];
    bool distinct = ls != nullptr && ls != ctx->lanes[0].stream && ls != ctx->s_h2d && ls != ctx->s_d2h;
    for (int j = 1; j < i; ++j) distinct &= ls != ctx->lanes[j].stream;
    if (!distinct) {
      delete ctx;
      return fail(nullptr, HYDRA_E_INVAL, "lane_streams must hold a distinct non-null stream for every lane above 0");
    }
    ctx->lanes[i].stream = ls;
  }
  if ((desc->flags & HYDRA_FLAG_D2H_MEMCPY) && (desc->flags & HYDRA_FLAG_D2H_KERNEL)) {
    delete ctx;
    return fail(nullptr, HYDRA_E_INVAL, "HYDRA_FLAG_D2H_MEMCPY and HYDRA_FLAG_D2H_KERNEL exclude each other");
  }
  if (desc->copy_blocks < 0 || desc->copy_blocks > 1024 || desc->prefetch_depth < 0) {
    delete ctx;
    return fail(nullptr, HYDRA_E_INVAL, "copy_blocks must be 0..1024 and prefetch_depth >= 0");
  }
  if (!ctx->dry && (desc->flags & HYDRA_FLAG_TIMING)) {
    ctx->prof = prof_create();
    prof_activate(ctx->prof);
  }
  if (!ctx->dry && (desc->flags & HYDRA_FLAG_OVERLAP)) ctx->tracer = trace_create();
  ctx->gate_on = !ctx->dry && (desc->flags & HYDRA_FLAG_GRAPHS) != 0;
  if (!ctx->dry) {
    // one coordinator thread per copy direction issues every promote and write-back (with or without a staging area)
    if (desc->stage_threads < 0 || desc->stage_threads > 16) {
      hydra_destroy(ctx);
      return fail(nullptr, HYDRA_E_INVAL, "stage_threads must be 0..16");
    }
    std::string perr;
    ctx->pager = pager_create(ctx, desc->stage, desc->stage_bytes, desc->stage_threads > 0 ? desc->stage_threads - 1 : 4, &perr);
    if (!ctx->pager) {
      hydra_destroy(ctx);
      return fail(nullptr, HYDRA_E_INVAL, perr);
    }
  }
  *out = ctx;
  return HYDRA_OK;
}

hydra_status hydra_destroy(hydra_ctx *ctx) {
  if (!ctx) return HYDRA_OK;
  if (!ctx->dry) {
    if (ctx->pager) (void)pager_drain(ctx->pager, nullptr);
    if (ctx->rounder) {  // its jobs wait for tickets of the staging tier: before that goes
      worker_destroy(ctx->rounder);
      ctx->rounder = nullptr;
    }
    if (ctx->pager) {
      pager_destroy(ctx->pager);
      ctx->pager = nullptr;
    }
    for (hydra_ctx::Lane &ln : ctx->lanes) (void)hipStreamSynchronize(ln.stream);
    (void)hipStreamSynchronize(ctx->s_h2d);
    (void)hipStreamSynchronize(ctx->s_d2h);
    prof_destroy(ctx->prof);
    trace_destroy(ctx->tracer);
    for (auto &kv : ctx->graphs)
      if (kv.second.exec) (void)hipGraphExecDestroy(kv.second.exec);
    for (Slot &s : ctx->slots) {
      if (s.ev_loaded) (void)hipEventDestroy(s.ev_loaded);
      if (s.ev_compute) (void)hipEventDestroy(s.ev_compute);
      if (s.ev_spilled) (void)hipEventDestroy(s.ev_spilled);
    }
  }
  for (Model *m : ctx->models) {
    if (!ctx->dry) destroy_model_events(m);
    delete m;
  }
  delete ctx;
  return HYDRA_OK;
}

hydra_status hydra_sync(hydra_ctx *ctx) {
  if (!ctx) return fail(nullptr, HYDRA_E_INVAL, "null context");
  if (ctx->dry) return HYDRA_OK;
  hydra_status st = drain_copies(ctx);
  if (st) return st;
  HYDRA_HIP(ctx, hipStreamSynchronize(ctx->s_h2d));
  for (hydra_ctx::Lane &ln : ctx->lanes) HYDRA_HIP(ctx, hipStreamSynchronize(ln.stream));
  HYDRA_HIP(ctx, hipStreamSynchronize(ctx->s_d2h));
  if (ctx->rounder) worker_drain(ctx->rounder);  // the bf16 host copies are current when the call returns
  return HYDRA_OK;
}

const char *hydra_last_error(const hydra_ctx *ctx) { return ctx ? ctx->err.c_str() : global_error(); }

hydra_status hydra_get_stats(hydra_ctx *ctx, hydra_stats *out) {
  if (!ctx || !out) return fail(ctx, HYDRA_E_INVAL, "null argument");
  *out = ctx->stats;
  out->n_graph_launches = ctx->graph_launches;
  return HYDRA_OK;
}

hydra_status hydra_register_model(hydra_ctx *ctx, const hydra_model_desc *desc, const hydra_host_state *host,
                                  int32_t *model_id) {
  if (!ctx || !desc || !host || !model_id) return fail(ctx, HYDRA_E_INVAL, "null argument");
  if (ctx->planned) return fail(ctx, HYDRA_E_STATE, "models must be registered before the first shard call");
  if (!host->master || !host->adam_m || !host->adam_v) return fail(ctx, HYDRA_E_INVAL, "null host state array");
  if (!host->batch_stage) return fail(ctx, HYDRA_E_INVAL, "null batch staging array");
  if ((ctx->init.flags & HYDRA_FLAG_CKPT_SPILL) && !host->ckpt)
    return fail(ctx, HYDRA_E_INVAL, "checkpoint spilling needs a host checkpoint array");
  Model *m = new Model();
  std::string err;
  hydra_status st = build_shape(desc, &m->sh, &err);
  if (st != HYDRA_OK) {
    delete m;
    return fail(ctx, st, err);
  }
  m->desc = *desc;
  m->host = *host;
  // each state array on its own: page-locked memory is copied directly, ordinary memory through the staging area
  // (what the driver lets a process page-lock may cover some of a model's arrays and not the others)
  auto kind_of = [&](const void *p) { return ctx->dry || page_locked(p) ? CopyPlan::SEG_PINNED : CopyPlan::SEG_PAGEABLE; };
  m->kind_w = kind_of(host->master);
  m->kind_m = kind_of(host->adam_m);
  m->kind_v = kind_of(host->adam_v);
  m->pageable = m->kind_w == CopyPlan::SEG_PAGEABLE;
  m->dtype = desc->dtype;
  m->fwd_bf16 = host->work_bf16 != nullptr && desc->dtype == DT_BF16;
  m->kind_work = m->fwd_bf16 ? kind_of(host->work_bf16) : CopyPlan::SEG_PINNED;
  if ((m->kind_w || m->kind_m || m->kind_v || m->kind_work) && !ctx->init.stage) {
    delete m;
    return fail(ctx, HYDRA_E_INVAL, "a state array is not page-locked and hydra_init was given no staging area");
  }
  m->host_dev = *host;  // entries of arrays in ordinary memory are never used
  if ((!m->kind_w && (st = mapped_pointer(ctx, host->master, "master", &m->host_dev.master, true))) ||
      (!m->kind_m && (st = mapped_pointer(ctx, host->adam_m, "adam_m", &m->host_dev.adam_m, true))) ||
      (!m->kind_v && (st = mapped_pointer(ctx, host->adam_v, "adam_v", &m->host_dev.adam_v, true))) ||
      (st = mapped_pointer(ctx, host->ckpt, "ckpt", &m->host_dev.ckpt))) {
    delete m;
    return st;
  }
  if (m->fwd_bf16 && !ctx->dry) {
    // a page-locked master is rounded into the copy by a thread of the library after each write-back
    if (!m->pageable && !ctx->rounder) ctx->rounder = worker_create();
    host_round_bf16_threads(host->work_bf16, host->master, (size_t)m->sh.n_params, 8);
  }
  m->round_ticket.assign(m->sh.S + 2, 0);
  const ModelShape &s = m->sh;
  const uint64_t act = (uint64_t)s.Mt * s.d * 4;  // boundary tensors hold all micro-batches
  const bool spill = (ctx->init.flags & HYDRA_FLAG_CKPT_SPILL) != 0;
  auto take = [&](uint64_t bytes) -> char * { return arena_take(ctx, bytes); };
  bool ok = true;
  ok &= (m->tok = (int32_t *)take(s.Mt * 4)) != nullptr;
  ok &= (m->tgt = (int32_t *)take(s.Mt * 4)) != nullptr;
  m->ckpt.assign(s.S + 1, nullptr);
  if (spill) {
    float *pp[2];
    ok &= (pp[0] = (float *)take(act)) != nullptr;
    ok &= (pp[1] = (float *)take(act)) != nullptr;
    for (int b = 0; b <= s.S; ++b) m->ckpt[b] = pp[b & 1];
  } else {
    for (int b = 0; b <= s.S; ++b) ok &= (m->ckpt[b] = (float *)take(act)) != nullptr;
  }
  ok &= (m->dbound[0] = (float *)take(act)) != nullptr;
  ok &= (m->dbound[1] = (float *)take(act)) != nullptr;
  ok &= (m->dlogits = take((uint64_t)s.Mt * s.Vpad * dt_size(m->dtype))) != nullptr;
  ok &= (m->row_loss = (float *)take(s.Mt * 4)) != nullptr;
  ok &= (m->loss = (float *)take(256)) != nullptr;
  if (s.tie) ok &= (m->tied_g = (float *)take((uint64_t)s.V * s.d * 4)) != nullptr;
  if (!ok) {
    delete m;
    return fail(ctx, HYDRA_E_NOMEM, "device arena too small for the model's activations");
  }
  m->slot_of.assign(s.S + 2, -1);
  m->wb_pending.assign(s.S + 2, 0);
  m->wb_ticket.assign(s.S + 2, 0);
  m->lane = (int)(ctx->models.size() % ctx->lanes.size());
  m->stage = host->batch_stage;
  if (!ctx->dry) {
    hipPointerAttribute_t at;
    if (hipPointerGetAttributes(&at, m->stage) != hipSuccess || at.type != hipMemoryTypeHost) {
      (void)hipGetLastError();
      delete m;
      return fail(ctx, HYDRA_E_INVAL, "batch_stage is not page-locked host memory");
    }
    m->ev_wb.assign(s.S + 2, nullptr);
    st = HYDRA_OK;
    for (int i = 0; i < 2 && !st; ++i)
      (void)((st = make_event(ctx, &m->ev_stage[i])) || (st = make_event(ctx, &m->ev_ckpt_d2h[i])) ||
             (st = make_event(ctx, &m->ev_ckpt_h2d[i])));
    if (!st) st = make_event(ctx, &m->ev_last_compute);
    for (hipEvent_t &e : m->ev_wb)
      if (!st) st = make_event(ctx, &e);
    if (st) {  // release what was created: the model is not registered
      destroy_model_events(m);
      delete m;
      return st;
    }
  }
  *model_id = (int32_t)ctx->models.size();
  ctx->models.push_back(m);
  return HYDRA_OK;
}

hydra_status hydra_set_batch(hydra_ctx *ctx, int32_t model, const int32_t *tokens, const int32_t *targets) {
  hydra_status st = check_model(ctx, model, 0);
  if (st) return st;
  if (!tokens || !targets) return fail(ctx, HYDRA_E_INVAL, "null token / target array");
  Model *m = ctx->models[model];
  const int64_t M = m->sh.Mt;
  int64_t nv = 0;
  for (int64_t i = 0; i < M; ++i) {
    if (tokens[i] < 0 || tokens[i] >= m->sh.V) return fail(ctx, HYDRA_E_INVAL, "token id out of range");
    if (targets[i] >= m->sh.V) return fail(ctx, HYDRA_E_INVAL, "target id out of range");
    nv += targets[i] >= 0;
  }
  if (nv == 0) return fail(ctx, HYDRA_E_INVAL, "minibatch has no valid target");
  const int si = m->stage_idx;
  int32_t *st_tok = m->stage + (size_t)si * 2 * M, *st_tgt = st_tok + M;
  if (!ctx->dry && m->stage_used[si]) HYDRA_HIP(ctx, hipEventSynchronize(m->ev_stage[si]));
  memcpy(st_tok, tokens, M * 4);
  memcpy(st_tgt, targets, M * 4);
  if (!ctx->dry) {
    hipStream_t cs = ctx->lanes[m->lane].stream;
    HYDRA_HIP(ctx, hipMemcpyAsync(m->tok, st_tok, M * 4, hipMemcpyHostToDevice, cs));
    HYDRA_HIP(ctx, hipMemcpyAsync(m->tgt, st_tgt, M * 4, hipMemcpyHostToDevice, cs));
    HYDRA_HIP(ctx, hipEventRecord(m->ev_stage[si], cs));
    m->stage_used[si] = true;
  }
  m->stage_idx ^= 1;
  m->n_valid = nv;
  m->t += 1;
  m->next_fwd = 0;
  m->next_bwd = -1;
  m->logits_valid = false;
  return HYDRA_OK;
}

hydra_status hydra_shard_load_async(hydra_ctx *ctx, int32_t model, int32_t shard, int32_t what) {
  hydra_status st = check_model(ctx, model, shard);
  if (st) return st;
  if (!(what & HYDRA_LOAD_PARAMS) || (what & ~3)) return fail(ctx, HYDRA_E_INVAL, "bad 'what' for load");
  if ((st = ensure_planned(ctx))) return st;
  Model *m = ctx->models[model];
  const int64_t off = m->sh.shard_off[shard], cnt = m->sh.shard_off[shard + 1] - off;
  if ((st = pager_check(ctx))) return st;
  ctx->stats.n_loads++;
  Slot *sl = slot_for(ctx, model, shard);
  CopyPlan plan;
  plan.trace_tag = model << 16 | shard;
  const int host_kind = m->kind_w;
  if (!sl) {
    int free_i = -1;
    for (size_t i = 0; i < ctx->slots.size(); ++i)
      if (ctx->slots[i].model < 0) { free_i = (int)i; break; }
    if (free_i < 0) {
      ctx->stats.n_loads--;
      return fail(ctx, HYDRA_E_NOSLOT, "no free shard buffer");
    }
    sl = &ctx->slots[free_i];
    sl->model = model; sl->shard = shard;
    sl->has_params = sl->has_opt = sl->wb_valid = sl->wbt_valid = sl->grads_valid = sl->dirty = sl->tied_valid = false;
    sl->has_fwd = false;
    sl->wb_seq = 0;
    m->slot_of[shard] = free_i;
    // the buffer's previous occupant must be done with it
    if (sl->compute_pending) plan.waits.push_back(sl->ev_compute);
    if (sl->spill_pending) {
      plan.waits.push_back(sl->ev_spilled);
      if (sl->spill_ticket) plan.d2h_tickets.push_back(sl->spill_ticket);
    }
    sl->compute_pending = sl->spill_pending = false;
  } else if ((sl->has_params && (sl->has_opt || !(what & HYDRA_LOAD_OPT))) || (sl->has_fwd && !(what & HYDRA_LOAD_OPT))) {
    ctx->stats.n_load_hits++;
  }
  // a promote for a forward visit of a block shard of a model with a bf16 host copy carries that copy and the fp32
  // vectors; every other promote the fp32 master
  bool fwd_only = m->fwd_bf16 && shard >= 1 && shard <= m->sh.S && !(what & HYDRA_LOAD_OPT);
  if (fwd_only && !sl->has_params && !sl->has_fwd && !m->pageable && !ctx->dry && m->round_ticket[shard]) {
    // Page-locked state: the host job that rounds the shard's last write-back must have finished.  The calling
    // thread waits for it - at most until the device has caught up with that write-back, which lies a whole
    // backward and forward pass of enqueued work behind for all but the first block shards of a pass.
    worker_wait(ctx->rounder, m->round_ticket[shard]);
    m->round_ticket[shard] = 0;
    if (m->round_broken.load()) fwd_only = false;
  }
  const bool need_master = !sl->has_params && !fwd_only, need_fwd = fwd_only && !sl->has_params && !sl->has_fwd;
  // the host arrays of a shard are read only after its last write-back has landed (the buffer it was written
  // back from may be a different one)
  if ((need_master || need_fwd || ((what & HYDRA_LOAD_OPT) && !sl->has_opt)) && m->wb_pending[shard]) {
    if (!ctx->dry) plan.waits.push_back(m->ev_wb[shard]);
    if (m->wb_ticket[shard]) plan.d2h_tickets.push_back(m->wb_ticket[shard]);
    m->wb_pending[shard] = 0;
  }
  if (need_master) {
    plan.segs.push_back({sl->w, m->host.master + off, nullptr, (size_t)cnt * 4, host_kind});
    plan.trace_bytes += (uint64_t)cnt * 4;
    sl->has_params = sl->has_fwd = true;
  }
  if (need_fwd) {
    plan.segs.push_back({sl->wb, m->host.work_bf16 + off, nullptr, (size_t)cnt * 2, m->kind_work});
    plan.trace_bytes += (uint64_t)cnt * 2;
    // the vectors of a block lie in four runs between its matrices (the last one runs on into the next block's first)
    const BlockOffsets &o = m->sh.bo;
    const int64_t d = m->sh.d, F = m->sh.F;
    auto run = [&](int64_t at, int64_t n) {
      plan.segs.push_back({sl->w + at, m->host.master + off + at, nullptr, (size_t)n * 4, host_kind});
      plan.trace_bytes += (uint64_t)n * 4;
    };
    for (int j = 0; j < m->sh.k; ++j) {
      const int64_t base = (int64_t)j * o.size;
      if (j == 0) run(base + o.ln1_g, 2 * d);
      run(base + o.b_qkv, 3 * d);
      run(base + o.b_o, 3 * d);
      run(base + o.b_fc, F);
      run(base + o.b_proj, j + 1 < m->sh.k ? 3 * d : d);
    }
    sl->has_fwd = sl->wb_valid = true;
  }
  if (m->sh.tie && shard == m->sh.S + 1 && !sl->tied_valid) {
    // tied LM head: the buffer keeps a copy of wte behind the final LayerNorm's parameters.  Taken from the EMBED
    // shard's buffer when that is resident (it may hold an update not yet written back), else from the host.
    const uint64_t bytes = (uint64_t)m->sh.V * m->sh.d * 4;
    Slot *e = slot_for(ctx, model, 0);
    if (e && e->has_params) {
      if (e->compute_pending) plan.waits.push_back(e->ev_compute);
      plan.segs.push_back({sl->w + 2 * m->sh.d, e->w, nullptr, (size_t)bytes, CopyPlan::SEG_DEVICE});
    } else {
      if (m->wb_pending[0]) {
        if (!ctx->dry) plan.waits.push_back(m->ev_wb[0]);
        if (m->wb_ticket[0]) plan.d2h_tickets.push_back(m->wb_ticket[0]);
        m->wb_pending[0] = 0;
      }
      plan.segs.push_back({sl->w + 2 * m->sh.d, m->host.master, nullptr, (size_t)bytes, host_kind});
      plan.trace_bytes += bytes;
    }
    sl->tied_valid = true;
    sl->wb_valid = false;
  }
  if ((what & HYDRA_LOAD_OPT) && !sl->has_opt) {
    plan.segs.push_back({sl->m, m->host.adam_m + off, nullptr, (size_t)cnt * 4, m->kind_m});
    plan.segs.push_back({sl->v, m->host.adam_v + off, nullptr, (size_t)cnt * 4, m->kind_v});
    plan.trace_bytes += (uint64_t)cnt * 8;
    sl->has_opt = true;
  }
  ctx->stats.bytes_h2d += plan.trace_bytes;
  if (!plan.segs.empty()) {
    plan.records.push_back(sl->ev_loaded);
    sl->need_wait_load = true;
  }
  if (ctx->dry || (plan.segs.empty() && plan.waits.empty())) return HYDRA_OK;
  uint64_t ticket = 0;
  if ((st = issue_plan(ctx, PQ_H2D, plan, &ticket))) return st;
  if (!plan.segs.empty()) sl->load_ticket = ticket;
  return HYDRA_OK;
}

hydra_status hydra_shard_spill(hydra_ctx *ctx, int32_t model, int32_t shard, int32_t what) {
  hydra_status st = check_model(ctx, model, shard);
  if (st) return st;
  if (!(what & 3) || (what & ~3)) return fail(ctx, HYDRA_E_INVAL, "bad 'what' for spill");
  if ((st = ensure_planned(ctx))) return st;
  Model *m = ctx->models[model];
  Slot *sl = slot_for(ctx, model, shard);
  if (!sl) return fail(ctx, HYDRA_E_STATE, "shard is not resident");
  if ((what & HYDRA_SPILL_EVICT) && sl->dirty && !(what & HYDRA_SPILL_WRITEBACK))
    return fail(ctx, HYDRA_E_STATE, "evicting a shard whose updated state was not written back");
  const int64_t off = m->sh.shard_off[shard], cnt = m->sh.shard_off[shard + 1] - off;
  if ((st = pager_check(ctx))) return st;
  const bool writeback = (what & HYDRA_SPILL_WRITEBACK) && sl->dirty;
  const bool poison = (what & HYDRA_SPILL_EVICT) && (ctx->init.flags & HYDRA_FLAG_POISON);
  if (writeback || poison) {
    CopyPlan plan;
    plan.trace_tag = model << 16 | shard;
    plan.tokens_per_visit = m->sh.Mt;
    // after the last task that used the buffer
    if (sl->compute_pending) plan.waits.push_back(sl->ev_compute);
    if (writeback) {
      plan.segs.push_back({m->host.master + off, sl->w, m->host_dev.master + off, (size_t)cnt * 4, m->kind_w});
      plan.segs.push_back({m->host.adam_m + off, sl->m, m->host_dev.adam_m + off, (size_t)cnt * 4, m->kind_m});
      plan.segs.push_back({m->host.adam_v + off, sl->v, m->host_dev.adam_v + off, (size_t)cnt * 4, m->kind_v});
      plan.trace_bytes = (uint64_t)cnt * 12;
      // the host's bf16 copy follows the master: state in ordinary memory is rounded by the staging tier's threads on
      // its way out of the ring (page-locked state: by a host job once the write-back has landed, below)
      if (m->fwd_bf16 && m->pageable && shard >= 1 && shard <= m->sh.S)
        plan.segs[plan.segs.size() - 3].rounded = m->host.work_bf16 + off;
      if (!ctx->dry) plan.records.push_back(m->ev_wb[shard]);
    }
    if (poison) {  // on the d2h stream: behind the write-back
      plan.poison = true;
      plan.poison_base = sl->base;
      plan.poison_words = (int64_t)(ctx->slot_bytes / 4);
    }
    if (!ctx->dry) plan.records.push_back(sl->ev_spilled);
    uint64_t ticket = 0;
    if ((st = issue_plan(ctx, PQ_D2H, plan, &ticket))) return st;
    sl->spill_pending = true;
    sl->spill_ticket = ticket;
    if (writeback && m->fwd_bf16 && !m->pageable && !ctx->dry && shard >= 1 && shard <= m->sh.S) {
      // The write-back's event may be recorded by the staging tier's thread (a context with a staging area issues
      // every plan there): wait for that, then for the event, then round.  The shard's next write-back is a whole
      // minibatch away, so the event is not recorded again before this job has waited for it.
      Pager *pg = ctx->pager;
      hipEvent_t ev = m->ev_wb[shard];
      uint16_t *dst = m->host.work_bf16 + off;
      const float *src = m->host.master + off;
      m->round_ticket[shard] = worker_submit(ctx->rounder, [ctx, pg, ticket, ev, dst, src, cnt, m] {
        if (pg && ticket) pager_wait(pg, PQ_D2H, ticket);
        if (wait_event(ctx, ev) != hipSuccess) {
          (void)hipGetLastError();
          m->round_broken.store(true);
          return;
        }
        host_round_bf16_threads(dst, src, (size_t)cnt, 4);
      });
    }
    if (writeback) {
      m->wb_pending[shard] = 1;
      m->wb_ticket[shard] = ticket;
      sl->wb_seq = ++ctx->wb_counter;
      sl->dirty = false;
      ctx->stats.bytes_d2h += plan.trace_bytes;
      ctx->stats.n_writebacks++;
    }
  }
  if (what & HYDRA_SPILL_EVICT) {
    m->slot_of[shard] = -1;
    sl->model = sl->shard = -1;
    sl->has_params = sl->has_opt = sl->wb_valid = sl->wbt_valid = sl->grads_valid = sl->tied_valid = false;
    sl->has_fwd = false;
    ctx->stats.n_evictions++;
  }
  return HYDRA_OK;
}

// Checkpoints through host DRAM (HYDRA_FLAG_CKPT_SPILL): the device holds a ping-pong pair of boundary buffers, and
// boundary b lives in buffer b & 1 while it is needed.  The backward visit of shard sh reads boundary sh - 1.  The
// last two boundaries are still on the device when the backward pass starts; every other one is fetched from the
// host right after the backward visit that last needed the buffer it goes into has been enqueued (shard sh + 1).
static hydra_status promote_checkpoint(hydra_ctx *ctx, Model *m, int b) {
  if (b < 0 || m->ckpt_in_buf[b & 1] == b) return HYDRA_OK;
  const uint64_t bytes = (uint64_t)m->sh.Mt * m->sh.d * 4;
  if (!ctx->dry) {
    if (m->compute_pending) HYDRA_HIP(ctx, hipStreamWaitEvent(ctx->s_h2d, m->ev_last_compute, 0));
    if (m->ckpt_d2h_pending[b & 1]) HYDRA_HIP(ctx, hipStreamWaitEvent(ctx->s_h2d, m->ev_ckpt_d2h[b & 1], 0));
    const int tr = trace_begin(ctx, TRACE_H2D, ctx->s_h2d);
    HYDRA_HIP(ctx, hipMemcpyAsync(m->ckpt[b], m->host.ckpt + (uint64_t)b * m->sh.Mt * m->sh.d, bytes,
                                  hipMemcpyHostToDevice, ctx->s_h2d));
    trace_end(ctx, tr, ctx->s_h2d, bytes);
    HYDRA_HIP(ctx, hipEventRecord(m->ev_ckpt_h2d[b & 1], ctx->s_h2d));
  }
  m->ckpt_h2d_pending[b & 1] = true;
  m->ckpt_in_buf[b & 1] = b;
  ctx->stats.bytes_h2d += bytes;
  return HYDRA_OK;
}

// common entry of the three compute calls: the shard must have been promoted
static hydra_status begin_task(hydra_ctx *ctx, int model, int shard, Slot **out, bool forward = false) {
  hydra_status st = check_model(ctx, model, shard);
  if (st) return st;
  if ((st = ensure_planned(ctx))) return st;
  Slot *sl = slot_for(ctx, model, shard);
  if (!sl || !(forward ? sl->has_fwd : sl->has_params)) return fail(ctx, HYDRA_E_STATE, "shard was not loaded");
  if (ctx->models[model]->sh.tie && shard == ctx->models[model]->sh.S + 1 && !sl->tied_valid)
    return fail(ctx, HYDRA_E_STATE, "tied LM head: load the shard again after the embedding shard's update");
  if (sl->need_wait_load) {
    if (!ctx->dry) {
      // with a staging tier the promote is issued by another thread: the event can be waited for once it is recorded
      if (ctx->pager && sl->load_ticket) pager_wait(ctx->pager, PQ_H2D, sl->load_ticket);
      if ((st = pager_check(ctx))) return st;
      HYDRA_HIP(ctx, hipStreamWaitEvent(ctx->lanes[ctx->models[model]->lane].stream, sl->ev_loaded, 0));
    }
    sl->need_wait_load = false;
  }
  *out = sl;
  return HYDRA_OK;
}

static hydra_status end_task(hydra_ctx *ctx, Model *m, Slot *sl, int tr) {
  if (!ctx->dry) {
    trace_end(ctx, tr, ctx->lanes[m->lane].stream, 0);
    HYDRA_HIP(ctx, hipEventRecord(sl->ev_compute, ctx->lanes[m->lane].stream));
    HYDRA_HIP(ctx, hipEventRecord(m->ev_last_compute, ctx->lanes[m->lane].stream));
  }
  sl->compute_pending = true;
  sl->last_use = ++ctx->use_counter;
  m->compute_pending = true;
  ctx->stats.n_tasks++;
  return HYDRA_OK;
}

hydra_status hydra_shard_forward(hydra_ctx *ctx, int32_t model, int32_t shard) {
  Slot *sl = nullptr;
  hydra_status st = begin_task(ctx, model, shard, &sl, true);
  if (st) return st;
  Model *m = ctx->models[model];
  if (m->t == 0) return fail(ctx, HYDRA_E_STATE, "no minibatch set");
  if (shard != m->next_fwd) return fail(ctx, HYDRA_E_STATE, "forward visits must follow shard order");
  const bool spill = (ctx->init.flags & HYDRA_FLAG_CKPT_SPILL) != 0;
  const int S = m->sh.S;
  if (spill && shard <= S && !ctx->dry && m->ckpt_d2h_pending[shard & 1]) {
    // the ping-pong buffer about to be overwritten may still be on its way to the host
    HYDRA_HIP(ctx, hipStreamWaitEvent(ctx->lanes[m->lane].stream, m->ev_ckpt_d2h[shard & 1], 0));
  }
  const int tr = ctx->dry ? -1 : trace_begin(ctx, TRACE_COMPUTE, ctx->lanes[m->lane].stream, model << 16 | shard);
  if (!ctx->dry && (st = exec_forward(ctx, m, sl, shard))) return st;
  if ((st = end_task(ctx, m, sl, tr))) return st;
  if (spill && shard <= S) {
    const uint64_t bytes = (uint64_t)m->sh.Mt * m->sh.d * 4;
    if (!ctx->dry) {
      HYDRA_HIP(ctx, hipStreamWaitEvent(ctx->s_d2h, m->ev_last_compute, 0));
      const uint64_t eo = (uint64_t)shard * m->sh.Mt * m->sh.d;
      const int tr = trace_begin(ctx, TRACE_D2H, ctx->s_d2h);
      hydra_status cs = copy_d2h(ctx, m->host.ckpt + eo, m->host_dev.ckpt + eo, m->ckpt[shard], bytes, m->sh.Mt);
      if (cs) return cs;
      trace_end(ctx, tr, ctx->s_d2h, bytes);
      HYDRA_HIP(ctx, hipEventRecord(m->ev_ckpt_d2h[shard & 1], ctx->s_d2h));
    }
    m->ckpt_d2h_pending[shard & 1] = true;
    ctx->stats.bytes_d2h += bytes;
  }
  m->next_fwd = shard + 1;
  if (shard <= S) m->ckpt_in_buf[shard & 1] = shard;
  if (shard == S + 1) {
    m->next_bwd = S + 1;
    m->logits_valid = true;
  }
  return HYDRA_OK;
}

hydra_status hydra_shard_backward(hydra_ctx *ctx, int32_t model, int32_t shard) {
  Slot *sl = nullptr;
  hydra_status st = begin_task(ctx, model, shard, &sl);
  if (st) return st;
  Model *m = ctx->models[model];
  if (m->next_bwd < 0) return fail(ctx, HYDRA_E_STATE, "backward before the forward pass has finished");
  if (shard != m->next_bwd) return fail(ctx, HYDRA_E_STATE, "backward visits must follow reverse shard order");
  const bool ckpt_spill = (ctx->init.flags & HYDRA_FLAG_CKPT_SPILL) != 0;
  if (ckpt_spill && shard >= 1) {
    const int pb = (shard - 1) & 1;
    if ((st = promote_checkpoint(ctx, m, shard - 1))) return st;  // a no-op unless the caller skipped a visit's prefetch
    if (m->ckpt_h2d_pending[pb] && !ctx->dry) HYDRA_HIP(ctx, hipStreamWaitEvent(ctx->lanes[m->lane].stream, m->ev_ckpt_h2d[pb], 0));
    m->ckpt_h2d_pending[pb] = false;
  }
  const int tr = ctx->dry ? -1 : trace_begin(ctx, TRACE_COMPUTE, ctx->lanes[m->lane].stream, model << 16 | shard);
  if (!ctx->dry && (st = exec_backward(ctx, m, sl, shard))) return st;
  sl->grads_valid = true;
  if ((st = end_task(ctx, m, sl, tr))) return st;
  m->next_bwd = shard - 1;  // -1 after the embedding shard: minibatch finished
  // the boundary the next backward visit (shard - 1) reads goes into the buffer this visit's predecessor used
  if (ckpt_spill && shard - 1 >= 1 && (st = promote_checkpoint(ctx, m, shard - 2))) return st;
  return HYDRA_OK;
}

hydra_status hydra_shard_adam_step(hydra_ctx *ctx, int32_t model, int32_t shard) {
  Slot *sl = nullptr;
  hydra_status st = begin_task(ctx, model, shard, &sl);
  if (st) return st;
  Model *m = ctx->models[model];
  if (!sl->grads_valid) return fail(ctx, HYDRA_E_STATE, "no gradients: run the backward visit first");
  if (!sl->has_opt) return fail(ctx, HYDRA_E_STATE, "Adam state not resident: load with HYDRA_LOAD_OPT");
  if (sl->spill_pending && !ctx->dry) {
    // a write-back of this buffer (the shard stayed resident after it) may still be reading w, m and v; its event
    // can be waited for once the coordinator thread has recorded it
    if (ctx->pager && sl->spill_ticket) pager_wait(ctx->pager, PQ_D2H, sl->spill_ticket);
    if ((st = pager_check(ctx))) return st;
    HYDRA_HIP(ctx, hipStreamWaitEvent(ctx->lanes[m->lane].stream, sl->ev_spilled, 0));
  }
  const int tr = ctx->dry ? -1 : trace_begin(ctx, TRACE_COMPUTE, ctx->lanes[m->lane].stream, model << 16 | shard);
  if (!ctx->dry && (st = exec_adam(ctx, m, sl, shard))) return st;
  sl->grads_valid = false;
  sl->dirty = true;
  if (m->sh.tie && shard == 0) {  // the HEAD shard's copy of wte is now out of date
    Slot *hs = slot_for(ctx, model, m->sh.S + 1);
    if (hs) hs->tied_valid = hs->wb_valid = false;
  }
  ctx->stats.n_tasks--;  // the optimizer step belongs to the backward task
  return end_task(ctx, m, sl, tr);
}

hydra_status hydra_get_loss(hydra_ctx *ctx, int32_t model, float *loss) {
  hydra_status st = check_model(ctx, model, 0);
  if (st) return st;
  if (!loss) return fail(ctx, HYDRA_E_INVAL, "null output");
  Model *m = ctx->models[model];
  if (m->next_fwd != m->sh.S + 2) return fail(ctx, HYDRA_E_STATE, "the HEAD forward visit has not run");
  if (ctx->dry) {
    *loss = 0.f;
    return HYDRA_OK;
  }
  HYDRA_HIP(ctx, hipStreamSynchronize(ctx->lanes[m->lane].stream));
  HYDRA_HIP(ctx, hipMemcpy(loss, m->loss, 4, hipMemcpyDeviceToHost));
  return HYDRA_OK;
}

hydra_status hydra_read_device(hydra_ctx *ctx, int32_t model, int32_t shard, int32_t which, void *host_dst,
                               uint64_t bytes) {
  hydra_status st = check_model(ctx, model, shard);
  if (st) return st;
  if (!host_dst) return fail(ctx, HYDRA_E_INVAL, "null destination");
  if ((st = ensure_planned(ctx))) return st;
  Model *m = ctx->models[model];
  const ModelShape &s = m->sh;
  const uint64_t act = (uint64_t)s.Mt * s.d * 4;
  if (!ctx->dry && (st = hydra_sync(ctx))) return st;
  const void *src = nullptr;
  uint64_t need = 0;
  switch (which) {
    case HYDRA_RD_LOGITS: {
      if (!m->logits_valid || ctx->lanes[m->lane].logits_owner != model)
        return fail(ctx, HYDRA_E_STATE, "logits of this model are no longer held");
      need = (uint64_t)s.M * s.V * 4;
      if (bytes != need) return fail(ctx, HYDRA_E_INVAL, "size mismatch");
      if (!ctx->dry)
        HYDRA_HIP(ctx, hipMemcpy2D(host_dst, (size_t)s.V * 4, ctx->lanes[m->lane].logits, (size_t)s.Vpad * 4, (size_t)s.V * 4, s.M,
                                   hipMemcpyDeviceToHost));
      return HYDRA_OK;
    }
    case HYDRA_RD_GRADS:
    case HYDRA_RD_PARAMS:
    case HYDRA_RD_ADAM_M:
    case HYDRA_RD_ADAM_V: {
      Slot *sl = slot_for(ctx, model, shard);
      if (!sl) return fail(ctx, HYDRA_E_STATE, "shard is not resident");
      if (which == HYDRA_RD_GRADS && !sl->grads_valid) return fail(ctx, HYDRA_E_STATE, "no gradients held");
      if ((which == HYDRA_RD_ADAM_M || which == HYDRA_RD_ADAM_V) && !sl->has_opt)
        return fail(ctx, HYDRA_E_STATE, "Adam state not resident");
      if (which == HYDRA_RD_PARAMS && !sl->has_params) return fail(ctx, HYDRA_E_STATE, "fp32 master not resident");
      src = which == HYDRA_RD_GRADS ? sl->g : which == HYDRA_RD_PARAMS ? sl->w : which == HYDRA_RD_ADAM_M ? sl->m : sl->v;
      need = (uint64_t)(s.shard_off[shard + 1] - s.shard_off[shard]) * 4;
      break;
    }
    case HYDRA_RD_CKPT:
      if (shard > s.S) return fail(ctx, HYDRA_E_INVAL, "no boundary after the HEAD shard");
      src = m->ckpt[shard];
      need = act;
      break;
    case HYDRA_RD_DBOUND:
      src = m->dbound[m->dcur];
      need = act;
      break;
    default:
      return fail(ctx, HYDRA_E_INVAL, "unknown 'which'");
  }
  if (bytes != need) return fail(ctx, HYDRA_E_INVAL, "size mismatch");
  if (!ctx->dry) HYDRA_HIP(ctx, hipMemcpy(host_dst, src, need, hipMemcpyDeviceToHost));
  return HYDRA_OK;
}

}  // extern "C"
