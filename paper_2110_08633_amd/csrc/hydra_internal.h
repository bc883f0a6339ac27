// Internal host-side structures of the library (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <functional>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/hydra.h"
#include "kernels.h"

namespace hydra {

struct Profiler;
Profiler *prof_create();
void prof_destroy(Profiler *p);
void prof_activate(Profiler *p);
void prof_collect(Profiler *p, hipEvent_t base);
void prof_reset(Profiler *p);

// swap / compute overlap trace (HYDRA_FLAG_OVERLAP)
struct Tracer;
enum { TRACE_COMPUTE = 0, TRACE_H2D = 1, TRACE_D2H = 2 };
Tracer *trace_create();
void trace_destroy(Tracer *t);

// staging tier for host state that is not page-locked (pager.cpp)
struct Pager;
struct HostWorker;
enum { PQ_H2D = 0, PQ_D2H = 1 };

struct TensorInfo {
  std::string name;
  int64_t off, rows, cols;
  int shard;
};

// Offsets (in elements, relative to the start of a block) of a block's tensors.
struct BlockOffsets {
  int64_t ln1_g, ln1_b, w_qkv, b_qkv, w_o, b_o, ln2_g, ln2_b, w_fc, b_fc, w_proj, b_proj, size;
};

struct ModelShape {
  int L, d, H, F, V, T, B, k, S, dh;
  int nm;        // micro-batches per minibatch
  int64_t M;     // tokens per micro-batch
  int64_t Mt;    // tokens per minibatch = nm * M
  int64_t Vpad;  // leading dimension of logits / dlogits
  BlockOffsets bo;
  int64_t n_params;
  std::vector<int64_t> shard_off;  // S+3 entries
  int64_t max_shard;               // largest shard as held in a shard buffer, elements
  int tie;                         // LM head tied to the token embedding
};

hydra_status build_shape(const hydra_model_desc *d, ModelShape *out, std::string *err);
void list_tensors(const ModelShape &s, std::vector<TensorInfo> *out);

struct Slot {
  char *base = nullptr;
  float *w = nullptr, *m = nullptr, *v = nullptr, *g = nullptr;
  bf16_t *wb = nullptr;   // bf16 working copy of the shard, same layout as the master (dx products; the LM head's
                          // copy is kept transposed here)
  bf16_t *wbt = nullptr;  // block shards: every weight matrix transposed ([out, in]) at the matrix's own offset, so
                          // that forward products have both operands contraction-contiguous
  int model = -1, shard = -1;
  bool has_params = false, has_opt = false, wb_valid = false, wbt_valid = false, grads_valid = false, dirty = false;
  bool has_fwd = false;  // what a forward visit reads is resident (bf16 copy wb and the fp32 vectors in w), be the fp32
                         // master resident or not
  bool need_wait_load = false;  // a copy into this slot was enqueued since the compute stream last waited
  hipEvent_t ev_loaded = nullptr, ev_compute = nullptr, ev_spilled = nullptr;
  bool compute_pending = false, spill_pending = false;
  bool tied_valid = false;  // HEAD shard of a tied model: the buffer's copy of wte is current
  uint64_t last_use = 0;  // value of the context's task counter when a task last ran on this buffer
  uint64_t load_ticket = 0, spill_ticket = 0;  // staging tier: the jobs that issue the buffer's last promote / write-back
  uint64_t wb_seq = 0;    // position of the buffer's last write-back in the order write-backs were enqueued (0: none
                          // since it was filled); the d2h stream works in that order, so a smaller value is free earlier
};

struct Model {
  hydra_model_desc desc;
  hydra_host_state host;
  hydra_host_state host_dev;  // device-side mappings of the same page-locked arrays
  ModelShape sh;
  int dtype;
  int lane = 0;
  // device state carved from the arena
  int32_t *tok = nullptr, *tgt = nullptr;
  std::vector<float *> ckpt;  // boundary b -> buffer (ping-pong pair when checkpoints are spilled)
  float *dbound[2] = {nullptr, nullptr};
  int dcur = 0;
  void *dlogits = nullptr;
  float *row_loss = nullptr, *loss = nullptr;
  // pinned staging for tokens / targets (two minibatches deep)
  int32_t *stage = nullptr;
  int stage_idx = 0;
  hipEvent_t ev_stage[2] = {nullptr, nullptr};
  bool stage_used[2] = {false, false};
  hipEvent_t ev_ckpt_d2h[2] = {nullptr, nullptr};
  bool ckpt_d2h_pending[2] = {false, false};
  hipEvent_t ev_ckpt_h2d[2] = {nullptr, nullptr};
  bool ckpt_h2d_pending[2] = {false, false};
  int ckpt_in_buf[2] = {-1, -1};  // spilled checkpoints: boundary index held by each ping-pong buffer
  hipEvent_t ev_last_compute = nullptr;
  bool compute_pending = false;
  int64_t t = 0;        // minibatches handed over = Adam step of the current minibatch
  int64_t n_valid = 0;  // targets >= 0 in the current minibatch
  int next_fwd = 0;     // next forward visit expected
  int next_bwd = -1;    // next backward visit expected (-1: none)
  bool logits_valid = false;
  std::vector<int> slot_of;  // shard -> slot index or -1
  float *tied_g = nullptr;   // tied LM head: its part of the wte gradient [V,d], from HEAD backward to EMBED backward
  std::vector<hipEvent_t> ev_wb;   // per shard: last write-back to the host arrays
  std::vector<char> wb_pending;
  std::vector<uint64_t> wb_ticket;  // staging tier: job of the shard's last write-back
  bool pageable = false;            // the master is ordinary host memory: its copies go through the staging ring, and
                                    // the ring's threads keep the bf16 host copy
  int kind_w = 0, kind_m = 0, kind_v = 0, kind_work = 0;  // CopyPlan::SEG_PINNED / SEG_PAGEABLE of each host array
  bool fwd_bf16 = false;            // the host keeps a bf16 rounding of the master (hydra_host_state.work_bf16):
                                    // promotes for forward visits of block shards carry that instead of the master
  std::vector<uint64_t> round_ticket;  // page-locked state: per shard, the host job that rounds its last write-back
                                       // into work_bf16 (0: none pending)
  std::atomic<bool> round_broken{false};  // such a job could not wait for its write-back: the copy is no longer used
};

}  // namespace hydra

struct hydra_ctx {
  hydra_init_desc init;
  bool dry = false;
  bool planned = false;
  hipStream_t s_h2d = nullptr, s_d2h = nullptr;
  // Compute lanes: each has its own stream and workspace; a model always runs on lane (model id % lanes), so
  // tasks of different models may overlap on the device while every model's own tasks stay in order.
  struct Lane {
    hipStream_t stream = nullptr;  // the caller's
    char *ws = nullptr;
    int logits_owner = -1;    // model whose logits the lane's workspace still holds
    float *logits = nullptr;
  };
  std::vector<Lane> lanes;
  char *arena = nullptr;
  uint64_t arena_bytes = 0, arena_used = 0;
  std::vector<hydra::Model *> models;
  std::vector<hydra::Slot> slots;
  uint64_t slot_bytes = 0, slot_elems = 0;
  uint64_t ws_bytes = 0;  // workspace per lane (one task at a time runs on a lane)
  hydra_stats stats;
  uint64_t use_counter = 0;
  uint64_t wb_counter = 0;  // write-backs enqueued so far
  hydra::Profiler *prof = nullptr;  // per-kernel event timing (HYDRA_FLAG_TIMING)
  hydra::Tracer *tracer = nullptr;  // promote / write-back / task intervals (HYDRA_FLAG_OVERLAP)
  hydra::Pager *pager = nullptr;    // staging ring and its threads (hydra_init_desc.stage)
  hydra::HostWorker *rounder = nullptr;  // rounds written-back page-locked masters into their bf16 host copies
  // With HYDRA_FLAG_GRAPHS: the calling thread holds this while it captures a shard visit, and the library's threads
  // take it around every HIP call they make (and poll events instead of blocking in the runtime).  A capture was
  // invalidated whenever one of them called into the runtime meanwhile, whatever capture mode either side declared.
  std::mutex hip_gate;
  bool gate_on = false;
  // captured block-shard visits (HYDRA_FLAG_GRAPHS); key: model, shard, phase, shard buffer, boundary-gradient parity
  struct GraphEntry {
    int seen = 0;  // visits run so far without a graph
    bool failed = false;
    hipGraphExec_t exec = nullptr;
  };
  std::map<uint64_t, GraphEntry> graphs;
  uint64_t graph_launches = 0;
  std::string err;
};

namespace hydra {

hydra_status fail(hydra_ctx *ctx, hydra_status code, const std::string &msg);
hydra_status hipfail(hydra_ctx *ctx, hipError_t e, const char *what);
void set_global_error(const std::string &msg);
const char *global_error();
hydra_status ensure_planned(hydra_ctx *ctx);
Slot *slot_for(hydra_ctx *ctx, int model, int shard);
// device -> host copy on the d2h stream: own copy kernel, or hipMemcpyAsync with HYDRA_FLAG_D2H_MEMCPY
hydra_status copy_d2h(hydra_ctx *ctx, void *host_dst, void *host_dst_mapped, const void *src, size_t bytes,
                      int64_t tokens_per_visit);

// opens / closes an interval of the overlap trace on stream s (no-ops without HYDRA_FLAG_OVERLAP; idx < 0 ignored)
int trace_begin(hydra_ctx *ctx, int kind, hipStream_t s, int tag = 0);  // tag: model << 16 | shard
void trace_end(hydra_ctx *ctx, int idx, hipStream_t s, uint64_t bytes);

// executor (exec.cpp): enqueue the kernels of one visit on the compute stream
hydra_status exec_forward(hydra_ctx *ctx, Model *mm, Slot *sl, int shard);
hydra_status exec_backward(hydra_ctx *ctx, Model *mm, Slot *sl, int shard);
hydra_status exec_adam(hydra_ctx *ctx, Model *mm, Slot *sl, int shard);
uint64_t workspace_need(const ModelShape &s, int dtype);
// staging tier
Pager *pager_create(hydra_ctx *ctx, void *stage, uint64_t stage_bytes, int helpers, std::string *err);
void pager_destroy(Pager *p);
uint64_t pager_submit(Pager *p, int which, std::function<hydra_status()> job);  // returns the job's ticket
void pager_wait(Pager *p, int which, uint64_t ticket);                          // until that job has run
hydra_status pager_error(Pager *p, std::string *text);
hydra_status pager_drain(Pager *p, std::string *text);
hydra_status pager_h2d(Pager *p, void *dst_dev, const void *src_host, size_t bytes);
hydra_status pager_d2h(Pager *p, void *dst_host, const void *src_dev, size_t bytes, int64_t tokens_per_visit,
                       uint16_t *rounded);
// a thread that runs host-side jobs in submission order; tickets count from 1 (0: nothing to wait for)
HostWorker *worker_create();
void worker_destroy(HostWorker *w);  // after running what is still queued
uint64_t worker_submit(HostWorker *w, std::function<void()> job);
void worker_wait(HostWorker *w, uint64_t ticket);
void worker_drain(HostWorker *w);
// scope in which a library thread may call the HIP runtime (no-op unless the context replays graphs)
struct HipGate {
  hydra_ctx *c;
  explicit HipGate(hydra_ctx *ctx) : c(ctx) { if (c->gate_on) c->hip_gate.lock(); }
  ~HipGate() { if (c->gate_on) c->hip_gate.unlock(); }
  HipGate(const HipGate &) = delete;
  HipGate &operator=(const HipGate &) = delete;
};
// a library thread's wait for an event: hipEventSynchronize, or polling under the gate
hipError_t wait_event(hydra_ctx *ctx, hipEvent_t e);
// fp32 -> bf16 on the host with the device casts' rounding
void host_round_bf16(uint16_t *dst, const float *src, size_t n);
void host_round_bf16_threads(uint16_t *dst, const float *src, size_t n, int threads);
hydra_status drain_copies(hydra_ctx *ctx);
// device address of the current GPU's static scratch array (hydra_op_layernorm_bwd_static)
hydra_status static_scratch(float **out);

}  // namespace hydra

#define HYDRA_HIP(ctx, call)                                     \
  do {                                                           \
    hipError_t e__ = (call);                                     \
    if (e__ != hipSuccess) return hydra::hipfail(ctx, e__, #call); \
  } while (0)
