/*
 * hydra.h - C ABI of the MI355X (gfx950) library for spilled, shard-alternated
 * training of several GPT-2-style decoders on one GPU.
 *
 * The method (paper, Section 2.3 "Spilling" and Section 2.4 "Shard Alternator
 * Parallelism"): a model is cut into shards - contiguous runs of layers - whose
 * parameters live in host DRAM.  A shard is promoted to GPU memory, executed,
 * and demoted again; each shard is visited twice per minibatch (forward, then
 * backward).  Only the activation at a shard boundary is kept between visits;
 * the backward visit recomputes the shard's forward from it.  While one shard
 * executes, the next one - possibly of another model - is prefetched into a
 * second buffer (double buffering).  After every shard task the Sharded-LRTF
 * scheduler picks the model with the longest remaining time.
 *
 * Conventions
 *  - All functions return hydra_status (0 = ok, <0 = error).  Nothing aborts
 *    and no exception crosses the boundary; hydra_last_error() gives text.
 *  - The CALLER owns all memory and all streams: one device arena
 *    (sub-allocated by the library, never freed by it), the page-locked host
 *    arrays of every model including the staging area of its token batches,
 *    and the compute / copy streams.  The library allocates neither device nor
 *    page-locked memory and creates no stream; what it creates are HIP events
 *    (and HIP graphs with HYDRA_FLAG_GRAPHS), destroyed by hydra_destroy.
 *  - Every hydra_shard_* call only enqueues work on the streams given to
 *    hydra_init; ordering between streams is by events on the device.
 *  - The library reads no environment variable.
 *  - Each declaration below names the passage of the paper it follows; calls
 *    marked "plumbing" exist for the caller's convenience (set-up, inspection,
 *    measurement) and follow no passage.
 *  - Shards of a model: 0 = EMBED (wte, wpe); 1..S = runs of layers_per_shard
 *    blocks; S+1 = HEAD (final LayerNorm, LM head, loss).
 *  - Canonical flat parameter layout (fp32, row-major, matrices are [in,out]
 *    with y = x*W + b):
 *      EMBED  wte[V,d] wpe[T,d]
 *      block  ln1_g[d] ln1_b[d] w_qkv[d,3d] b_qkv[3d] w_o[d,d] b_o[d]
 *             ln2_g[d] ln2_b[d] w_fc[d,F] b_fc[F] w_proj[F,d] b_proj[d]
 *      HEAD   lnf_g[d] lnf_b[d] w_lm[d,V]
 *    One shard is one contiguous range, so a promote/demote is one large copy
 *    per state array.
 *  - Decoder mathematics (the paper only names "GPT-2", Section 3): pre-LN
 *    blocks, LayerNorm eps 1e-5 with biased variance, scores scaled by
 *    1/sqrt(d/H), causal mask with masked probabilities exactly 0, tanh-form
 *    GELU, no bias on the LM head, untied LM head, no dropout, loss = mean
 *    cross-entropy over positions with target >= 0, Adam without weight decay.
 *  - Shape limits: d, F, T multiples of 8; d/H a multiple of 8; V arbitrary.
 */
#ifndef HYDRA_H
#define HYDRA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hydra_ctx hydra_ctx;
typedef struct hydra_sched hydra_sched;
typedef int32_t hydra_status;

enum {
  HYDRA_OK = 0,
  HYDRA_E_INVAL = -1,  /* bad argument (null pointer, unsupported shape, bad index) */
  HYDRA_E_NOSLOT = -2, /* no free shard buffer: spill something first              */
  HYDRA_E_STATE = -3,  /* call not valid in the shard's / model's current state    */
  HYDRA_E_HIP = -4,    /* a HIP call failed; text in hydra_last_error              */
  HYDRA_E_NOMEM = -5   /* device arena too small                                   */
};

/* hydra_init_desc.flags */
enum {
  HYDRA_FLAG_DRY_RUN = 1,    /* no HIP call is made: state machine, slot table and traces only (host tests) */
  HYDRA_FLAG_CKPT_SPILL = 2, /* boundary activations travel through host DRAM between visits (Section 2.3:   */
                             /* "intermediate data" is demoted too); the device keeps a ping-pong pair       */
  HYDRA_FLAG_POISON = 4,     /* fill a shard buffer with NaN patterns when it is freed                       */
  HYDRA_FLAG_TIMING = 8,     /* bracket every kernel launch with HIP events; read with hydra_kernel_stats    */
  HYDRA_FLAG_D2H_MEMCPY = 16, /* every write-back through hipMemcpyAsync.  Without this flag and without           */
                              /* HYDRA_FLAG_D2H_KERNEL: page-locked state goes back through hipMemcpyAsync, state   */
                              /* in ordinary memory (staging area) and spilled checkpoints through the library's   */
                              /* own copy kernel - what measured best for each                                     */
  HYDRA_FLAG_GRAPHS = 32,    /* block-shard visits are captured as HIP graphs on their second run with a given  */
                             /* shard buffer and replayed from then on (one graph launch instead of dozens of   */
                             /* kernel launches: the host is the bottleneck otherwise); ignored with TIMING     */
  HYDRA_FLAG_D2H_KERNEL = 128, /* every write-back through the library's own copy kernel (not with D2H_MEMCPY)    */
  HYDRA_FLAG_OVERLAP = 64    /* bracket every promote, write-back and shard task with a HIP event pair on its   */
                             /* own stream; read with hydra_overlap_stats                                       */
};

/* 'what' of hydra_shard_load_async */
enum {
  HYDRA_LOAD_PARAMS = 1, /* master weights only (forward visit)            */
  HYDRA_LOAD_OPT = 2     /* Adam m and v as well (backward visit: 1|2 = 3) */
};
/* 'what' of hydra_shard_spill */
enum {
  HYDRA_SPILL_WRITEBACK = 1, /* copy weights/m/v back to the host arrays if Adam changed them */
  HYDRA_SPILL_EVICT = 2      /* release the shard buffer                                       */
};
/* 'which' of hydra_read_device */
enum {
  HYDRA_RD_LOGITS = 0, /* fp32 [B*T, V] of the model's last HEAD forward (its last micro-batch) */
  HYDRA_RD_GRADS = 1,  /* fp32 gradients of a resident shard after its backward     */
  HYDRA_RD_PARAMS = 2, /* fp32 master weights of a resident shard                   */
  HYDRA_RD_ADAM_M = 3,
  HYDRA_RD_ADAM_V = 4,
  HYDRA_RD_CKPT = 5,   /* fp32 [n_micro*B*T, d]: output activation of shard 'shard' (0..S)  */
  HYDRA_RD_DBOUND = 6  /* fp32 [n_micro*B*T, d]: gradient w.r.t. the input of the last backward visit */
};

#define HYDRA_MAX_LANES 8

typedef struct {
  void *dev_arena;                 /* device pointer; one buffer the library carves up        */
  uint64_t dev_arena_bytes;
  uint64_t shard_buffer_cap_bytes; /* upper bound on memory used for shard buffers; 0 = none  */
  int32_t max_slots;               /* upper bound on the number of shard buffers; 0 = none    */
  int32_t flags;
  void *compute_stream;            /* hipStream_t handles; NULL = the null stream             */
  void *h2d_stream;
  void *d2h_stream;
  int32_t compute_lanes;           /* 0 or 1: every task on compute_stream.  n > 1: model i runs on lane i % n, so  */
                                   /* that tasks of different models overlap on the device; lane 0 is compute_stream */
  int32_t copy_blocks;             /* workgroups of the write-back copy kernel; 0 = chosen from the tokens a shard  */
                                   /* visit works on and the shard's size (48 down to 8: fewer the more compute     */
                                   /* there is to disturb and the longer promote and write-back run side by side)   */
  void *lane_streams[HYDRA_MAX_LANES - 1]; /* caller's streams (default priority) of lanes 1 .. compute_lanes - 1;  */
                                   /* distinct non-null handles (ignored with HYDRA_FLAG_DRY_RUN)                   */
  int32_t prefetch_depth;          /* how many tasks ahead hydra_sched_run promotes shards for; 0 = one (the paper's  */
                                   /* double buffering, Section 2.3); more only helps while buffers can be freed     */
  int32_t stage_threads;           /* host threads per direction that copy between ordinary memory and the staging   */
                                   /* area; 0 = 5                                                                     */
  void *stage;                     /* page-locked host memory (256-byte aligned, >= 16 MiB), or NULL.  With it, a     */
  uint64_t stage_bytes;            /* model's master / adam_m / adam_v may be ORDINARY (pageable) host memory: their  */
                                   /* promotes and write-backs then travel through this area chunk by chunk (host     */
                                   /* threads of the library copy between the arrays and the area, the copy streams   */
                                   /* between the area and the shard buffers) - for state larger than the driver lets */
                                   /* a process page-lock.  The area belongs to the library until hydra_destroy.     */
} hydra_init_desc;

typedef struct {
  int32_t n_layer, d_model, n_head, d_ff, vocab, seq, batch;
  int32_t layers_per_shard; /* must divide n_layer                                        */
  int32_t dtype;            /* 0 = fp32 compute; 1 = bf16 MFMA compute, fp32 master/Adam  */
  int32_t n_micro;          /* micro-batches of 'batch' samples per minibatch (0 counts as 1): every visit of  */
                            /* a shard runs all of them while the shard is resident and sums their gradients,  */
                            /* so one promotion serves n_micro * batch samples (paper Section 2.3 leaves the   */
                            /* work done per visit open; activation memory stays that of one micro-batch)      */
  int32_t tie_embeddings;   /* 0: own LM head matrix w_lm[d,V].  1: logits = z * wte^T; the HEAD shard then owns   */
                            /* only the final LayerNorm, keeps a device copy of wte while resident, and hands its   */
                            /* part of the wte gradient to the EMBED shard's backward visit                        */
  int32_t reserved;
  double lr, beta1, beta2, eps; /* Adam hyper-parameters of this model (doubles so that 1-beta is exact) */
} hydra_model_desc;

typedef struct {
  /* caller-owned host memory; must outlive the model.  Page-locked - except that master, adam_m, adam_v and
   * work_bf16 may each be ordinary memory when hydra_init was given a staging area: an array in ordinary memory
   * travels through that area, a page-locked one directly (so a caller can page-lock as many of a model's arrays
   * as the driver allows and leave the rest) */
  float *master;  /* [n_params] fp32, canonical flat layout */
  float *adam_m;  /* [n_params]                               */
  float *adam_v;  /* [n_params]                               */
  float *ckpt;    /* [(S+1) * n_micro*B*T * d] fp32; only read/written with HYDRA_FLAG_CKPT_SPILL, else may be NULL */
  int32_t *batch_stage; /* [4 * n_micro*B*T] int32: staging of two minibatches' token ids and targets on their   */
                        /* way to the device; contents belong to the library while the model is registered        */
  uint16_t *work_bf16;  /* optional (NULL: not used; ignored for dtype 0): [n_params] bf16, the master rounded to   */
                        /* nearest-even, same layout.  Written by the library only: from master at registration   */
                        /* and after every write-back of a block shard.  A forward visit multiplies by this        */
                        /* rounding of the weights in any case, so with the array present the promote for a        */
                        /* FORWARD visit of a block shard (Section 2.3) carries it (2 bytes per parameter) plus    */
                        /* the shard's fp32 vectors instead of the whole fp32 master (4 bytes per parameter);      */
                        /* results do not change by a bit.  Kept current by host threads of the library: those of  */
                        /* the staging area round a master in ordinary memory as they move it out of the area; a   */
                        /* page-locked master is rounded by a thread of its own once a write-back has landed, and  */
                        /* a promote call that needs the result waits for it.  Current for the caller after        */
                        /* hydra_sync.  The caller must not change master while the model is registered, or this   */
                        /* copy goes stale.                                                                        */
} hydra_host_state;

typedef struct {
  int64_t n_params;
  int64_t params_per_block; /* 12 d^2 + 13 d when F = 4d */
  int32_t n_block_shards;   /* S                          */
  int32_t n_shards;         /* S + 2                      */
  int32_t n_tensors;
  int32_t reserved;
} hydra_layout;

typedef struct {
  int32_t model, shard;
  int32_t phase; /* 0 = forward visit, 1 = backward visit (includes the shard's Adam step) */
  int32_t minibatch;
} hydra_task;

typedef struct {
  uint64_t bytes_h2d, bytes_d2h;   /* parameter / optimizer / checkpoint traffic enqueued  */
  uint64_t n_loads, n_load_hits;   /* promote requests, and those already resident        */
  uint64_t n_evictions, n_writebacks;
  uint64_t n_tasks;
  int32_t n_slots;
  int32_t reserved;
  uint64_t slot_bytes, workspace_bytes, model_state_bytes;
  uint64_t n_graph_launches;       /* block-shard visits replayed as HIP graphs (HYDRA_FLAG_GRAPHS)       */
  double host_promote_ms;          /* host time hydra_sched_run spent inside promote (evict + load) calls  */
  double host_writeback_ms;        /* ... inside the write-back calls that follow an Adam step             */
  double host_task_ms;             /* ... and inside the forward / backward / Adam calls (kernel launches) */
  double host_batch_ms;            /* ... and inside hydra_set_batch: token staging is two minibatches deep, so this is */
                                   /* where a host that runs more than two minibatches ahead waits for the device       */
} hydra_stats;

/* How far the shard swaps are hidden under compute (paper Section 2.3, double buffering), from HIP events
 * recorded with HYDRA_FLAG_OVERLAP since the last reset.  An interval runs from the moment its stream reaches the
 * operation (all waits before it satisfied) to its completion; "busy" times are lengths of unions of intervals. */
typedef struct {
  double wall_ms;         /* first interval start to last interval end                                  */
  double compute_ms;      /* some shard task (forward / backward / Adam) in flight on any compute lane: */
                          /* from its first kernel's start to its last kernel's end, gaps included      */
  double h2d_ms;          /* some promote in flight (weights, Adam state, spilled checkpoints)          */
  double d2h_ms;          /* some write-back in flight                                                  */
  double transfer_ms;     /* h2d or d2h in flight                                                       */
  double hidden_ms;       /* transfer in flight while a shard task is in flight                         */
  uint64_t bytes_h2d, bytes_d2h; /* bytes moved by the recorded intervals                                */
  uint64_t n_intervals;
  double kernel_ms;       /* with HYDRA_FLAG_TIMING as well: some kernel of a shard task executing      */
  double hidden_kernel_ms;/* ... and transfer in flight while one executes (0 without HYDRA_FLAG_TIMING) */
} hydra_overlap;

/* ---- context (plumbing) -------------------------------------------------- */
/* Creates a context over the caller's arena and streams.  With
 * HYDRA_FLAG_DRY_RUN the arena pointer may be any non-null value. */
hydra_status hydra_init(const hydra_init_desc *desc, hydra_ctx **out);
/* Waits for all streams, destroys the library's events and graphs.  Caller memory and streams are left alone. */
hydra_status hydra_destroy(hydra_ctx *ctx);
/* Blocks until all streams of the context are idle. */
hydra_status hydra_sync(hydra_ctx *ctx);
/* Text of the last error seen on this context (ctx may be NULL for errors of
 * functions that take no context). Never NULL. */
const char *hydra_last_error(const hydra_ctx *ctx);
/* Byte, task and buffer counters since hydra_init (plumbing; the swap traffic of Section 2.3 in numbers). */
hydra_status hydra_get_stats(hydra_ctx *ctx, hydra_stats *out);

/* Per-kernel timing (plumbing; context created with HYDRA_FLAG_TIMING): entry 'index' of
 * the table of kernels launched since the last reset - name, number of
 * launches, summed HIP-event time on the launching stream, and the summed
 * algorithmic flops and bytes of those launches.  Synchronises.  Returns 1 when
 * index is past the end. */
hydra_status hydra_kernel_stats(hydra_ctx *ctx, int32_t index, char name[64], uint64_t *launches,
                                double *total_ms, double *flops, double *bytes);
hydra_status hydra_kernel_stats_reset(hydra_ctx *ctx);
/* Swap / compute overlap (measures what Section 2.3's double buffering hides; context created with
 * HYDRA_FLAG_OVERLAP, HYDRA_E_STATE otherwise).  All three synchronise the context's streams first.  The reset
 * forgets all intervals recorded so far.  hydra_overlap_dump writes one line per interval to a text file (kind,
 * model, shard, start ms, end ms, bytes; kind "kernel" lines with HYDRA_FLAG_TIMING) for timeline studies. */
hydra_status hydra_overlap_stats(hydra_ctx *ctx, hydra_overlap *out);
hydra_status hydra_overlap_reset(hydra_ctx *ctx);
hydra_status hydra_overlap_dump(hydra_ctx *ctx, const char *path);

/* ---- layout (pure functions of the model description) -------------------
 * A shard is a contiguous run of layers (Section 2.2: a model is rewritten into shards); these calls give the
 * element ranges that promotes and demotes move. */
hydra_status hydra_model_layout(const hydra_model_desc *desc, hydra_layout *out);
/* Tensor 'index' (0..n_tensors-1) in canonical order: name ("wte", "h3.w_qkv",
 * "lnf_g", ...; at most 31 chars + NUL), element offset into the flat arrays,
 * rows and cols (cols = 1 for vectors), and the shard that owns it. */
hydra_status hydra_model_tensor(const hydra_model_desc *desc, int32_t index, char name[32],
                                int64_t *offset, int64_t *rows, int64_t *cols, int32_t *shard);
/* Element range [offset, offset+count) of a shard in the flat arrays. */
hydra_status hydra_shard_range(const hydra_model_desc *desc, int32_t shard, int64_t *offset, int64_t *count);

/* ---- models -------------------------------------------------------------- */
/* Registers a model (the paper's interface takes a list of models with their
 * training specifications, Section 2.1).  All models must be registered before
 * the first load / forward / scheduler call. */
hydra_status hydra_register_model(hydra_ctx *ctx, const hydra_model_desc *desc,
                                  const hydra_host_state *host, int32_t *model_id);
/* Hands the next minibatch of a model to the library: host int32
 * [n_micro*B, T] token ids in [0,V) and targets (id or -1 = ignore); the loss
 * is the mean over all valid targets of the minibatch.  Copied before
 * returning control of the arrays; advances the model's Adam step counter t. */
hydra_status hydra_set_batch(hydra_ctx *ctx, int32_t model, const int32_t *tokens, const int32_t *targets);

/* ---- shard tasks (paper Section 2.3) ------------------------------------- */
/* Promote (Section 2.3): start copying the shard's state from the host arrays into a free
 * shard buffer on the h2d stream.  Returns once the copies have been handed to the stream
 * (or, with a staging area, to the library's threads), not when they have finished; before
 * that the calling thread waits for what the promote depends on - the write-back that freed
 * the buffer, the shard's own last write-back - so the call may take as long as those still
 * need.  Already resident: only missing parts are fetched.  No free buffer: HYDRA_E_NOSLOT. */
hydra_status hydra_shard_load_async(hydra_ctx *ctx, int32_t model, int32_t shard, int32_t what);
/* Forward visit: reads the boundary activation at the shard's input, writes
 * the one at its output (EMBED reads the tokens; HEAD writes logits and loss). */
hydra_status hydra_shard_forward(hydra_ctx *ctx, int32_t model, int32_t shard);
/* Backward visit: recompute the shard's forward from its input checkpoint,
 * back-propagate the incoming boundary gradient, leave parameter gradients in
 * the shard buffer and the outgoing boundary gradient for the next visit. */
hydra_status hydra_shard_backward(hydra_ctx *ctx, int32_t model, int32_t shard);
/* Adam on the shard's parameters with the gradients left by the backward
 * visit; needs m and v resident (HYDRA_LOAD_OPT). */
hydra_status hydra_shard_adam_step(hydra_ctx *ctx, int32_t model, int32_t shard);
/* Demote: write back changed state on the d2h stream and/or release the buffer. */
hydra_status hydra_shard_spill(hydra_ctx *ctx, int32_t model, int32_t shard, int32_t what);

/* Loss of the model's last HEAD forward (plumbing; synchronises the model's compute stream). */
hydra_status hydra_get_loss(hydra_ctx *ctx, int32_t model, float *loss);
/* Copies device data to host memory for inspection (plumbing; synchronous). */
hydra_status hydra_read_device(hydra_ctx *ctx, int32_t model, int32_t shard, int32_t which,
                               void *host_dst, uint64_t bytes);

/* ---- Sharded-LRTF scheduler (paper Section 2.4) --------------------------- */
/* task_cost[m] points to 2*(S_m+2) integers: forward-visit cost of shards
 * 0..S+1, then backward-visit cost of shards 0..S+1.  The remaining time of a
 * model is the summed cost of its tasks not yet started; the next task comes
 * from the model with the largest remaining time, ties to the lowest index.
 * ctx may be NULL when only hydra_sched_next is used (decision only). With a
 * ctx, shapes are taken from the registered models model_ids[m]; without,
 * n_block_shards[m] gives S per model. */
hydra_status hydra_sched_create(hydra_ctx *ctx, int32_t n_models, const int32_t *model_ids,
                                const int32_t *n_block_shards, const int32_t *n_minibatches,
                                const int64_t *const *task_cost, hydra_sched **out);
hydra_status hydra_sched_destroy(hydra_sched *s);
/* Next decision; returns 1 (not an error) when all tasks have been handed out. */
hydra_status hydra_sched_next(hydra_sched *s, hydra_task *out);
/* Runs every remaining task: the shards of the following tasks are promoted
 * before task n is enqueued - hydra_init_desc.prefetch_depth tasks ahead (default one),
 * as long as buffers can be freed without touching a shard an earlier task needs -
 * and a shard's updated state is written back right after its Adam step.
 * tokens[m] / targets[m]: host int32 [n_minibatches[m], n_micro*B, T].  trace (may be
 * NULL) receives the executed order. Returns after everything is enqueued
 * (call hydra_sync to wait). */
hydra_status hydra_sched_run(hydra_sched *s, const int32_t *const *tokens, const int32_t *const *targets,
                             hydra_task *trace, int64_t trace_cap, int64_t *n_executed);

/* ---- partitioner and pilot pass (paper Section 2.2, Algorithm 1) ----------
 * The paper finds cut points by running layer after layer on the GPU until
 * memory runs out.  This library knows the device footprint of a shard in
 * closed form, so the same walk runs on the host: open a shard at layer 0;
 * when adding layer i to the open shard would exceed the bound, cut before i
 * and open a new shard with layer i. */

/* Device bytes a backward visit of a shard of n_layers blocks needs: its shard
 * buffer (fp32 weights, Adam m, v, gradients, bf16 working copy) plus the
 * visit's workspace (kept activations of the recomputation and scratch).
 * n_layers = 0: the larger of the EMBED / HEAD shards.  desc->n_layer and
 * desc->layers_per_shard are ignored. */
hydra_status hydra_shard_footprint(const hydra_model_desc *desc, int32_t n_layers, uint64_t *bytes);

/* Greedy walk over desc->n_layer blocks against mem_bound_bytes.  cuts (host,
 * capacity cuts_cap, may be NULL with cuts_cap 0) receives the first layer of
 * every shard, *n_shards their number, *layers_per_shard the largest divisor of
 * n_layer that is not above the shortest closed shard of the walk (the executor
 * runs equal shards; use it as desc->layers_per_shard).  HYDRA_E_NOMEM when a
 * single block, or the EMBED / HEAD shard, exceeds the bound.
 * desc->layers_per_shard is ignored. */
hydra_status hydra_partition(const hydra_model_desc *desc, uint64_t mem_bound_bytes, int32_t *cuts,
                             int32_t cuts_cap, int32_t *n_shards, int32_t *layers_per_shard);

/* Pilot pass: runs one minibatch (host int32 [n_micro*B, T] tokens / targets)
 * of a registered model shard by shard, each task alone on the device, twice
 * (the first round absorbs one-time costs such as code loading), and writes
 * the second round's measured duration in nanoseconds of the forward visits of shards
 * 0..S+1, then of the backward visits (with their Adam step) of shards 0..S+1,
 * to costs_ns (host, 2*(S+2) entries): the cost table hydra_sched_create takes.
 * Every update of the pass is discarded and the Adam step counter is left as it
 * was: the model's host arrays are not written.  Needs no updated state of the
 * model pending on the device (HYDRA_E_STATE otherwise); blocks until done. */
hydra_status hydra_pilot_costs(hydra_ctx *ctx, int32_t model, const int32_t *tokens, const int32_t *targets,
                               int64_t *costs_ns);

/* ---- single kernels, exposed for parity tests and roofline measurement ----
 * Plumbing: the paper names the architecture (GPT-2, Section 3) and none of its
 * operators; each call below is one operator of that decoder with the textbook
 * definition stated.  No call allocates; bad sizes, leading dimensions or dtypes
 * return HYDRA_E_INVAL before anything is launched.
 * All pointers are DEVICE pointers, 'stream' a hipStream_t (NULL = null
 * stream).  dtype: 0 = fp32 operands, 1 = bf16 operands (fp32 accumulate). */

/* C[M,N] = alpha * op(A) * op(B) (+ bias[N]) (+ resid[M,N]); ta = 0: A is [M,K]
 * row-major, 1: A is [K,M]; tb = 0: B is [N,K] row-major, 1: B is [K,N].
 * out_f32 / out_act (operand dtype) may each be NULL. Leading dimensions in
 * elements. */
hydra_status hydra_op_gemm(int32_t dtype, int32_t ta, int32_t tb, int32_t M, int32_t N, int32_t K,
                           float alpha, const void *A, int64_t lda, const void *B, int64_t ldb,
                           const float *bias, const float *resid, float *out_f32, void *out_act,
                           int64_t ldc, void *stream);
/* Fused Adam on n elements, step t >= 1 (update without weight decay; 1-beta
 * and the bias corrections 1-beta^t are evaluated in double on the host);
 * shadow_bf16 (bf16 copy of the new weights) may be NULL. */
hydra_status hydra_op_adam(float *w, float *m, float *v, const float *g, void *shadow_bf16, int64_t n,
                           double lr, double beta1, double beta2, double eps, int64_t t, void *stream);
/* Row LayerNorm: y (dtype) [M,d], mean/rstd fp32 [M]. */
hydra_status hydra_op_layernorm_fwd(int32_t dtype, const float *x, const float *gamma, const float *beta,
                                    void *y, float *mean, float *rstd, int32_t M, int32_t d, void *stream);
/* Backward of the row LayerNorm y = xhat * gamma + beta (the textbook formulas; the paper only names the
 * architecture, Section 3) in one pass over the rows: dx = dres + rstd * (dxhat - mean(dxhat) - xhat *
 * mean(dxhat * xhat)) with dxhat = dy * gamma, optionally its bf16 copy, and the column sums dgamma = sum_rows
 * dy * xhat, dbeta = sum_rows dy, dx_colsum = sum_rows dx (the bias gradient of a linear layer whose output
 * gradient dx is).  All pointers device; dy, x, dx fp32 [M,d]; mean, rstd fp32 [M] as written by
 * hydra_op_layernorm_fwd; gamma, dgamma, dbeta, dx_colsum fp32 [d]; dres (fp32 [M,d]), dx_bf16 and dx_colsum
 * may be NULL; scratch: fp32 [3 * d * ceil(M / 8)], overwritten.  d must be a multiple of 4 and at most 2048
 * (HYDRA_E_INVAL otherwise). */
hydra_status hydra_op_layernorm_bwd(const float *dy, const float *x, const float *mean, const float *rstd,
                                    const float *gamma, const float *dres, float *dx, void *dx_bf16,
                                    float *dgamma, float *dbeta, float *dx_colsum, float *scratch, int32_t M,
                                    int32_t d, void *stream);
/* hydra_op_layernorm_bwd for callers that cannot allocate device memory and cannot hand over a workspace either:
 * code under HIP graph capture, tight serving or training loops, harnesses that forbid hipMalloc.  Same arguments
 * minus 'scratch', same kernels, same results bit for bit; the partial column sums live in a fixed array of 2 Mi
 * floats (8 MiB) that every GPU the library runs on holds until the process ends.  3 * d * ceil(M / 8) must not
 * exceed 2 Mi (HYDRA_E_INVAL otherwise; d = 1024 allows M up to 5456 rows).  The call allocates nothing and frees
 * nothing (the array's address on a GPU is looked up by hydra_init, or by the first call on that GPU).  All calls
 * on one GPU share that GPU's array: calls that overlap in time on one GPU race - order them on one stream or with
 * events.  Nothing in the array needs clearing between calls (every partial sum read is written first by the same
 * call). */
hydra_status hydra_op_layernorm_bwd_static(const float *dy, const float *x, const float *mean, const float *rstd,
                                           const float *gamma, const float *dres, float *dx, void *dx_bf16,
                                           float *dgamma, float *dbeta, float *dx_colsum, int32_t M, int32_t d,
                                           void *stream);
/* Plumbing, host only (no HIP call): n floats at src -> their bf16 roundings at dst (round to nearest even, NaN stays
 * NaN), the rounding every cast of the device path uses and the one hydra_host_state.work_bf16 is kept with.  HOST
 * pointers; src and dst must not overlap. */
hydra_status hydra_host_round_bf16(uint16_t *dst, const float *src, int64_t n);
/* Causal softmax over rows of S fp32 [n_mat, T, T] -> P (dtype); entries j>i are 0. */
hydra_status hydra_op_softmax_causal(int32_t dtype, const float *S, void *P, int32_t n_mat, int32_t T,
                                     void *stream);
/* Cross-entropy: logits fp32 [M, ld] (first V columns valid), targets int32 [M];
 * writes row_loss fp32 [M] and dlogits (dtype) [M, ld] = (softmax - onehot)*inv_n. */
hydra_status hydra_op_cross_entropy(int32_t dtype, const float *logits, const int32_t *targets,
                                    float *row_loss, void *dlogits, int32_t M, int32_t V, int64_t ld,
                                    float inv_n, void *stream);

/* Fused causal self-attention, bf16 operands, head width dh = 64 or 128, T % 8 == 0, d = H*dh.
 * qkv [B*T, 3d] holds q | k | v (head h at columns h*dh of each part);
 * o [B*T, d] = softmax_{j<=i}(q_i.k_j / sqrt(dh)) v; lse fp32 [B*H*T] = log-sum-exp of every score row. */
hydra_status hydra_op_attention_fwd(const void *qkv, void *o, float *lse, int32_t B, int32_t H, int32_t T,
                                    int32_t dh, void *stream);
/* Its backward: d_o [B*T, d] -> dqkv [B*T, 3d] (dq | dk | dv); o and lse from the forward call;
 * dsum fp32 [B*H*T] is scratch the call fills. */
hydra_status hydra_op_attention_bwd(const void *qkv, const void *o, const void *d_o, const float *lse,
                                    float *dsum, void *dqkv, int32_t B, int32_t H, int32_t T, int32_t dh,
                                    void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HYDRA_H */
