// Partitioner and pilot pass (paper Section 2.2, Algorithm 1).
//
// The paper's partitioner discovers cut points by running layers on the GPU
// until an allocation fails.  Here the footprint of a shard of n blocks is a
// closed-form function of the model description (shard buffer plus the
// workspace of a backward visit), so the same greedy walk runs on the host:
// open a shard at layer 0; walk the layers; when adding layer i to the open
// shard would exceed the memory bound, cut before i and open a new shard with
// it.  The pilot pass (one minibatch, every task timed with HIP events, all
// updates discarded) yields the per-task costs the scheduler consumes.
#include <algorithm>
#include <vector>

#include "hydra_internal.h"

using namespace hydra;

namespace {

uint64_t up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

// bytes a visit of a shard of `elems` parameters needs in a shard buffer: fp32 weights, Adam m and v, gradients,
// and the two bf16 working copies (same formula as the buffer planner of the context)
uint64_t buffer_bytes(uint64_t elems) { return up(up(elems, 64) * 20, 256); }

}  // namespace

extern "C" {

hydra_status hydra_shard_footprint(const hydra_model_desc *desc, int32_t n_layers, uint64_t *bytes) {
  if (!desc || !bytes || n_layers < 0) {
    set_global_error("bad argument");
    return HYDRA_E_INVAL;
  }
  hydra_model_desc d = *desc;
  // shape of a model whose shards hold n_layers blocks (n_layers = 0: the EMBED / HEAD shards alone)
  d.layers_per_shard = n_layers > 0 ? n_layers : 1;
  d.n_layer = d.layers_per_shard;
  ModelShape s;
  std::string err;
  hydra_status st = build_shape(&d, &s, &err);
  if (st != HYDRA_OK) {
    set_global_error(err);
    return st;
  }
  const uint64_t embed = (uint64_t)s.V * s.d + (uint64_t)s.T * s.d, head = 2ull * s.d + (uint64_t)s.d * s.V;
  if (n_layers == 0) {
    // the workspace figure of a one-block model is the larger of a block visit and the head's visit (logits)
    *bytes = buffer_bytes(std::max(embed, head)) + workspace_need(s, d.dtype);
    return HYDRA_OK;
  }
  *bytes = buffer_bytes((uint64_t)n_layers * s.bo.size) + workspace_need(s, d.dtype);
  return HYDRA_OK;
}

hydra_status hydra_partition(const hydra_model_desc *desc, uint64_t mem_bound_bytes, int32_t *cuts, int32_t cuts_cap,
                             int32_t *n_shards, int32_t *layers_per_shard) {
  if (!desc || !n_shards || !layers_per_shard || (cuts_cap > 0 && !cuts)) {
    set_global_error("null argument");
    return HYDRA_E_INVAL;
  }
  if (desc->n_layer <= 0) {
    set_global_error("model has no layers");
    return HYDRA_E_INVAL;
  }
  uint64_t fixed = 0;
  hydra_status st = hydra_shard_footprint(desc, 0, &fixed);
  if (st != HYDRA_OK) return st;
  if (fixed > mem_bound_bytes) {
    set_global_error("memory bound is below the embedding / head shard");
    return HYDRA_E_NOMEM;
  }
  std::vector<int32_t> a;
  a.push_back(0);
  int start = 0, shortest_closed = desc->n_layer;
  for (int i = 0; i < desc->n_layer; ++i) {
    uint64_t need = 0;
    if ((st = hydra_shard_footprint(desc, i - start + 1, &need)) != HYDRA_OK) return st;
    if (need > mem_bound_bytes) {
      if (i == start) {
        set_global_error("memory bound is below a single block");
        return HYDRA_E_NOMEM;
      }
      shortest_closed = std::min(shortest_closed, i - start);
      a.push_back(i);
      start = i;
      --i;  // layer i is looked at again, now as the first layer of the new shard
    }
  }
  if ((int)a.size() > cuts_cap && cuts_cap > 0) {
    set_global_error("cut array too small");
    return HYDRA_E_INVAL;
  }
  for (size_t k = 0; k < a.size() && (int)k < cuts_cap; ++k) cuts[k] = a[k];
  *n_shards = (int32_t)a.size();
  // the executor runs equal shards: the largest divisor of the depth that no closed shard of the walk is below
  int k = std::min(shortest_closed, (int)desc->n_layer);
  while (desc->n_layer % k) --k;
  *layers_per_shard = k;
  return HYDRA_OK;
}

hydra_status hydra_pilot_costs(hydra_ctx *ctx, int32_t model, const int32_t *tokens, const int32_t *targets,
                               int64_t *costs_ns) {
  if (!ctx || !costs_ns) return fail(ctx, HYDRA_E_INVAL, "null argument");
  if (model < 0 || model >= (int32_t)ctx->models.size()) return fail(ctx, HYDRA_E_INVAL, "no such model");
  hydra_status st = ensure_planned(ctx);
  if (st) return st;
  Model *m = ctx->models[model];
  const int S = m->sh.S, n = S + 2;
  for (int s = 0; s < n; ++s) {
    Slot *sl = slot_for(ctx, model, s);
    if (sl && sl->dirty) return fail(ctx, HYDRA_E_STATE, "pilot pass needs the model's updated state written back first");
  }
  if (ctx->dry) {
    for (int i = 0; i < 2 * n; ++i) costs_ns[i] = 1;
    return HYDRA_OK;
  }
  const int64_t t_before = m->t;
  if ((st = hydra_set_batch(ctx, model, tokens, targets))) return st;
  hipStream_t cs = ctx->lanes[m->lane].stream;
  std::vector<hipEvent_t> ev(4 * n, nullptr);
  auto cleanup = [&]() {
    for (hipEvent_t e : ev)
      if (e) (void)hipEventDestroy(e);
  };
  for (auto &e : ev)
    if (hipEventCreate(&e) != hipSuccess) {
      cleanup();
      return fail(ctx, HYDRA_E_HIP, "hipEventCreate");
    }
  auto discard = [&](int s) -> hydra_status {
    Slot *sl = slot_for(ctx, model, s);
    if (sl) sl->dirty = false;  // the pilot's update is thrown away: the host arrays keep the state
    return hydra_shard_spill(ctx, model, s, HYDRA_SPILL_EVICT);
  };
  // two rounds over the same minibatch: the first absorbs one-time costs (code objects, first-touch of buffers),
  // the second is the one reported
  for (int round = 0; round < 2 && !st; ++round) {
    if (round == 1) {
      m->next_fwd = 0;
      m->next_bwd = -1;
    }
    for (int s = 0; s < n && !st; ++s) {
      if ((st = hydra_shard_load_async(ctx, model, s, HYDRA_LOAD_PARAMS))) break;
      if ((st = drain_copies(ctx))) break;  // (a staging tier issues the promote from its own thread)
      if (hipStreamSynchronize(ctx->s_h2d) != hipSuccess) { st = fail(ctx, HYDRA_E_HIP, "sync"); break; }
      (void)hipEventRecord(ev[2 * s], cs);
      if ((st = hydra_shard_forward(ctx, model, s))) break;
      (void)hipEventRecord(ev[2 * s + 1], cs);
      if (s != n - 1) st = discard(s);
    }
    for (int s = n - 1; s >= 0 && !st; --s) {
      if ((st = hydra_shard_load_async(ctx, model, s, HYDRA_LOAD_PARAMS | HYDRA_LOAD_OPT))) break;
      if ((st = drain_copies(ctx))) break;  // (a staging tier issues the promote from its own thread)
      if (hipStreamSynchronize(ctx->s_h2d) != hipSuccess) { st = fail(ctx, HYDRA_E_HIP, "sync"); break; }
      (void)hipEventRecord(ev[2 * n + 2 * s], cs);
      if ((st = hydra_shard_backward(ctx, model, s))) break;
      if ((st = hydra_shard_adam_step(ctx, model, s))) break;
      (void)hipEventRecord(ev[2 * n + 2 * s + 1], cs);
      st = discard(s);
    }
  }
  if (!st && hipStreamSynchronize(cs) != hipSuccess) st = fail(ctx, HYDRA_E_HIP, "sync");
  if (!st) st = hydra_sync(ctx);
  if (!st) {
    for (int i = 0; i < 2 * n; ++i) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, ev[2 * i], ev[2 * i + 1]) != hipSuccess) {
        st = fail(ctx, HYDRA_E_HIP, "hipEventElapsedTime");
        break;
      }
      costs_ns[i] = std::max<int64_t>(1, (int64_t)(ms * 1e6));
    }
  }
  cleanup();
  m->t = t_before;  // the pilot minibatch does not count as a training step
  m->next_fwd = 0;
  m->next_bwd = -1;
  m->logits_valid = false;
  return st;
}

}  // extern "C"
