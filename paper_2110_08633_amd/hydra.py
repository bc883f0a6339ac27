"""ctypes binding of include/hydra.h: same names, argument marshalling only.

The library is loaded from paper_2110_08633_amd/libhydra.so (built in-tree by
build.py).  There is no fallback: if the library is missing, import fails.
"""
from __future__ import annotations

import ctypes as C
import os

# torch owns the device memory and the streams handed to the library, so both must
# use the same HIP runtime: importing torch first makes libhydra.so bind to the
# libamdhip64 that torch has already loaded instead of bringing in a second copy.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhydra.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} not found: build it with `python -m paper_2110_08633_amd.build` "
                      "(there is no CPU fallback)")
lib = C.CDLL(LIB_PATH)

OK, E_INVAL, E_NOSLOT, E_STATE, E_HIP, E_NOMEM = 0, -1, -2, -3, -4, -5
FLAG_DRY_RUN, FLAG_CKPT_SPILL, FLAG_POISON, FLAG_TIMING, FLAG_D2H_MEMCPY, FLAG_GRAPHS, FLAG_OVERLAP = 1, 2, 4, 8, 16, 32, 64
FLAG_D2H_KERNEL = 128
LOAD_PARAMS, LOAD_OPT = 1, 2
SPILL_WRITEBACK, SPILL_EVICT = 1, 2
MAX_LANES = 8
RD_LOGITS, RD_GRADS, RD_PARAMS, RD_ADAM_M, RD_ADAM_V, RD_CKPT, RD_DBOUND = range(7)


class InitDesc(C.Structure):
    _fields_ = [("dev_arena", C.c_void_p), ("dev_arena_bytes", C.c_uint64),
                ("shard_buffer_cap_bytes", C.c_uint64), ("max_slots", C.c_int32), ("flags", C.c_int32),
                ("compute_stream", C.c_void_p), ("h2d_stream", C.c_void_p), ("d2h_stream", C.c_void_p),
                ("compute_lanes", C.c_int32), ("copy_blocks", C.c_int32),
                ("lane_streams", C.c_void_p * (MAX_LANES - 1)), ("prefetch_depth", C.c_int32), ("stage_threads", C.c_int32),
                ("stage", C.c_void_p), ("stage_bytes", C.c_uint64)]


class ModelDesc(C.Structure):
    _fields_ = [("n_layer", C.c_int32), ("d_model", C.c_int32), ("n_head", C.c_int32), ("d_ff", C.c_int32),
                ("vocab", C.c_int32), ("seq", C.c_int32), ("batch", C.c_int32), ("layers_per_shard", C.c_int32),
                ("dtype", C.c_int32), ("n_micro", C.c_int32), ("tie_embeddings", C.c_int32), ("reserved", C.c_int32),
                ("lr", C.c_double), ("beta1", C.c_double),
                ("beta2", C.c_double), ("eps", C.c_double)]


class HostState(C.Structure):
    _fields_ = [("master", C.c_void_p), ("adam_m", C.c_void_p), ("adam_v", C.c_void_p), ("ckpt", C.c_void_p),
                ("batch_stage", C.c_void_p), ("work_bf16", C.c_void_p)]


class Layout(C.Structure):
    _fields_ = [("n_params", C.c_int64), ("params_per_block", C.c_int64), ("n_block_shards", C.c_int32),
                ("n_shards", C.c_int32), ("n_tensors", C.c_int32), ("reserved", C.c_int32)]


class Task(C.Structure):
    _fields_ = [("model", C.c_int32), ("shard", C.c_int32), ("phase", C.c_int32), ("minibatch", C.c_int32)]


class Overlap(C.Structure):
    _fields_ = [("wall_ms", C.c_double), ("compute_ms", C.c_double), ("h2d_ms", C.c_double), ("d2h_ms", C.c_double),
                ("transfer_ms", C.c_double), ("hidden_ms", C.c_double), ("bytes_h2d", C.c_uint64),
                ("bytes_d2h", C.c_uint64), ("n_intervals", C.c_uint64), ("kernel_ms", C.c_double),
                ("hidden_kernel_ms", C.c_double)]


class Stats(C.Structure):
    _fields_ = [("bytes_h2d", C.c_uint64), ("bytes_d2h", C.c_uint64), ("n_loads", C.c_uint64),
                ("n_load_hits", C.c_uint64), ("n_evictions", C.c_uint64), ("n_writebacks", C.c_uint64),
                ("n_tasks", C.c_uint64), ("n_slots", C.c_int32), ("reserved", C.c_int32),
                ("slot_bytes", C.c_uint64), ("workspace_bytes", C.c_uint64), ("model_state_bytes", C.c_uint64),
                ("n_graph_launches", C.c_uint64), ("host_promote_ms", C.c_double), ("host_writeback_ms", C.c_double),
                ("host_task_ms", C.c_double), ("host_batch_ms", C.c_double)]


_P = C.POINTER
_vp, _i32, _i64, _u64, _f32, _f64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float, C.c_double

# name -> (restype, argtypes); every symbol declared in include/hydra.h
SIGNATURES = {
    "hydra_init": (_i32, [_P(InitDesc), _P(_vp)]),
    "hydra_destroy": (_i32, [_vp]),
    "hydra_sync": (_i32, [_vp]),
    "hydra_last_error": (C.c_char_p, [_vp]),
    "hydra_get_stats": (_i32, [_vp, _P(Stats)]),
    "hydra_kernel_stats": (_i32, [_vp, _i32, C.c_char_p, _P(_u64), _P(_f64), _P(_f64), _P(_f64)]),
    "hydra_kernel_stats_reset": (_i32, [_vp]),
    "hydra_overlap_stats": (_i32, [_vp, _P(Overlap)]),
    "hydra_overlap_reset": (_i32, [_vp]),
    "hydra_overlap_dump": (_i32, [_vp, C.c_char_p]),
    "hydra_model_layout": (_i32, [_P(ModelDesc), _P(Layout)]),
    "hydra_model_tensor": (_i32, [_P(ModelDesc), _i32, C.c_char_p, _P(_i64), _P(_i64), _P(_i64), _P(_i32)]),
    "hydra_shard_range": (_i32, [_P(ModelDesc), _i32, _P(_i64), _P(_i64)]),
    "hydra_register_model": (_i32, [_vp, _P(ModelDesc), _P(HostState), _P(_i32)]),
    "hydra_set_batch": (_i32, [_vp, _i32, _vp, _vp]),
    "hydra_shard_load_async": (_i32, [_vp, _i32, _i32, _i32]),
    "hydra_shard_forward": (_i32, [_vp, _i32, _i32]),
    "hydra_shard_backward": (_i32, [_vp, _i32, _i32]),
    "hydra_shard_adam_step": (_i32, [_vp, _i32, _i32]),
    "hydra_shard_spill": (_i32, [_vp, _i32, _i32, _i32]),
    "hydra_get_loss": (_i32, [_vp, _i32, _P(_f32)]),
    "hydra_read_device": (_i32, [_vp, _i32, _i32, _i32, _vp, _u64]),
    "hydra_sched_create": (_i32, [_vp, _i32, _P(_i32), _P(_i32), _P(_i32), _P(_P(_i64)), _P(_vp)]),
    "hydra_sched_destroy": (_i32, [_vp]),
    "hydra_op_attention_fwd": (_i32, [_vp, _vp, _vp, _i32, _i32, _i32, _i32, _vp]),
    "hydra_op_attention_bwd": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _vp]),
    "hydra_shard_footprint": (_i32, [_P(ModelDesc), _i32, _P(_u64)]),
    "hydra_partition": (_i32, [_P(ModelDesc), _u64, _P(_i32), _i32, _P(_i32), _P(_i32)]),
    "hydra_pilot_costs": (_i32, [_vp, _i32, _vp, _vp, _P(_i64)]),
    "hydra_sched_next": (_i32, [_vp, _P(Task)]),
    "hydra_sched_run": (_i32, [_vp, _P(_vp), _P(_vp), _P(Task), _i64, _P(_i64)]),
    "hydra_op_gemm": (_i32, [_i32, _i32, _i32, _i32, _i32, _i32, _f32, _vp, _i64, _vp, _i64, _vp, _vp, _vp, _vp,
                             _i64, _vp]),
    "hydra_op_adam": (_i32, [_vp, _vp, _vp, _vp, _vp, _i64, _f64, _f64, _f64, _f64, _i64, _vp]),
    "hydra_op_layernorm_fwd": (_i32, [_i32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp]),
    "hydra_op_layernorm_bwd": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp]),
    "hydra_op_layernorm_bwd_static": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp]),
    "hydra_host_round_bf16": (_i32, [_vp, _vp, _i64]),
    "hydra_op_softmax_causal": (_i32, [_i32, _vp, _vp, _i32, _i32, _vp]),
    "hydra_op_cross_entropy": (_i32, [_i32, _vp, _vp, _vp, _vp, _i32, _i32, _i64, _f32, _vp]),
}
for _n, (_r, _a) in SIGNATURES.items():
    _f = getattr(lib, _n)
    _f.restype, _f.argtypes = _r, _a


class HydraError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"hydra error {code}: {msg}")
        self.code = code


def _check(code, ctx=None):
    if code < 0:
        raise HydraError(code, lib.hydra_last_error(ctx).decode())
    return code


def _ptr(t):
    """Device / host pointer of a torch tensor or numpy array (or None)."""
    if t is None:
        return None
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    return t.ctypes.data


def _stream(s):
    if s is None:
        return None
    return s.cuda_stream if hasattr(s, "cuda_stream") else s


def model_desc(cfg, lr, dtype=None, beta1=0.9, beta2=0.999, eps=1e-8):
    """ModelDesc from a config dict with keys L, d, H, F, V, T, B, k, dtype and, optionally, n_micro."""
    dt = cfg["dtype"] if dtype is None else dtype
    return ModelDesc(cfg["L"], cfg["d"], cfg["H"], cfg["F"], cfg["V"], cfg["T"], cfg["B"], cfg["k"],
                     1 if dt == "bf16" else 0, int(cfg.get("n_micro", 1)), 1 if cfg.get("tie") else 0, 0,
                     lr, beta1, beta2, eps)


# ---- thin wrappers, same names as the C functions --------------------------

def hydra_init(arena, arena_bytes, compute_stream=None, h2d_stream=None, d2h_stream=None, flags=0,
               shard_buffer_cap_bytes=0, max_slots=0, compute_lanes=1, lane_streams=(), copy_blocks=0,
               prefetch_depth=0, stage=None, stage_bytes=0, stage_threads=0):
    lanes = (C.c_void_p * (MAX_LANES - 1))(*[_stream(x) for x in lane_streams])
    d = InitDesc(arena if isinstance(arena, int) else _ptr(arena), arena_bytes, shard_buffer_cap_bytes, max_slots,
                 flags, _stream(compute_stream), _stream(h2d_stream), _stream(d2h_stream), compute_lanes, copy_blocks,
                 lanes, prefetch_depth, stage_threads, stage if isinstance(stage, int) or stage is None else _ptr(stage),
                 stage_bytes)
    out = _vp()
    _check(lib.hydra_init(C.byref(d), C.byref(out)))
    return out


def hydra_destroy(ctx):
    return _check(lib.hydra_destroy(ctx))


def hydra_sync(ctx):
    return _check(lib.hydra_sync(ctx), ctx)


def hydra_last_error(ctx=None):
    return lib.hydra_last_error(ctx).decode()


def hydra_get_stats(ctx):
    s = Stats()
    _check(lib.hydra_get_stats(ctx, C.byref(s)), ctx)
    return {n: getattr(s, n) for n, _ in Stats._fields_ if not n.startswith("reserved")}


def hydra_kernel_stats(ctx):
    """List of dicts(name, launches, ms, flops, bytes) since the last reset."""
    out, i = [], 0
    while True:
        name = C.create_string_buffer(64)
        n, ms, fl, by = _u64(), _f64(), _f64(), _f64()
        r = _check(lib.hydra_kernel_stats(ctx, i, name, C.byref(n), C.byref(ms), C.byref(fl), C.byref(by)), ctx)
        if r == 1:
            return out
        out.append(dict(name=name.value.decode(), launches=n.value, ms=ms.value, flops=fl.value, bytes=by.value))
        i += 1


def hydra_kernel_stats_reset(ctx):
    return _check(lib.hydra_kernel_stats_reset(ctx), ctx)


def hydra_overlap_stats(ctx):
    """Dict of the interval-union lengths (ms) and bytes recorded since the last reset (HYDRA_FLAG_OVERLAP)."""
    o = Overlap()
    _check(lib.hydra_overlap_stats(ctx, C.byref(o)), ctx)
    return {n: getattr(o, n) for n, _ in Overlap._fields_}


def hydra_overlap_reset(ctx):
    return _check(lib.hydra_overlap_reset(ctx), ctx)


def hydra_overlap_dump(ctx, path):
    return _check(lib.hydra_overlap_dump(ctx, os.fsencode(path)), ctx)


def hydra_model_layout(desc):
    lay = Layout()
    _check(lib.hydra_model_layout(C.byref(desc), C.byref(lay)))
    return lay


def hydra_model_tensor(desc, index):
    name = C.create_string_buffer(32)
    off, rows, cols, shard = _i64(), _i64(), _i64(), _i32()
    _check(lib.hydra_model_tensor(C.byref(desc), index, name, C.byref(off), C.byref(rows), C.byref(cols),
                                  C.byref(shard)))
    return name.value.decode(), off.value, rows.value, cols.value, shard.value


def hydra_shard_range(desc, shard):
    off, cnt = _i64(), _i64()
    _check(lib.hydra_shard_range(C.byref(desc), shard, C.byref(off), C.byref(cnt)))
    return off.value, cnt.value


def hydra_register_model(ctx, desc, master, adam_m, adam_v, ckpt, batch_stage, work_bf16=None):
    hs = HostState(_ptr(master), _ptr(adam_m), _ptr(adam_v), _ptr(ckpt), _ptr(batch_stage), _ptr(work_bf16))
    mid = _i32()
    _check(lib.hydra_register_model(ctx, C.byref(desc), C.byref(hs), C.byref(mid)), ctx)
    return mid.value


def hydra_set_batch(ctx, model, tokens, targets):
    return _check(lib.hydra_set_batch(ctx, model, _ptr(tokens), _ptr(targets)), ctx)


def hydra_shard_load_async(ctx, model, shard, what):
    return _check(lib.hydra_shard_load_async(ctx, model, shard, what), ctx)


def hydra_shard_forward(ctx, model, shard):
    return _check(lib.hydra_shard_forward(ctx, model, shard), ctx)


def hydra_shard_backward(ctx, model, shard):
    return _check(lib.hydra_shard_backward(ctx, model, shard), ctx)


def hydra_shard_adam_step(ctx, model, shard):
    return _check(lib.hydra_shard_adam_step(ctx, model, shard), ctx)


def hydra_shard_spill(ctx, model, shard, what=SPILL_WRITEBACK | SPILL_EVICT):
    return _check(lib.hydra_shard_spill(ctx, model, shard, what), ctx)


def hydra_get_loss(ctx, model):
    v = _f32()
    _check(lib.hydra_get_loss(ctx, model, C.byref(v)), ctx)
    return v.value


def hydra_read_device(ctx, model, shard, which, host_array):
    """host_array: writable numpy array whose byte size is the size of the object read."""
    return _check(lib.hydra_read_device(ctx, model, shard, which, host_array.ctypes.data, host_array.nbytes), ctx)


def hydra_sched_create(ctx, model_ids, n_minibatches, task_costs, n_block_shards=None):
    """task_costs[m] = list of 2*(S+2) ints: forward costs of shards 0..S+1, then backward costs."""
    n = len(n_minibatches)
    ids = (_i32 * n)(*model_ids) if model_ids is not None else None
    nbs = (_i32 * n)(*n_block_shards) if n_block_shards is not None else None
    nmb = (_i32 * n)(*n_minibatches)
    rows = [(_i64 * len(c))(*c) for c in task_costs]
    tab = (_P(_i64) * n)(*[C.cast(r, _P(_i64)) for r in rows])
    out = _vp()
    _check(lib.hydra_sched_create(ctx, n, ids, nbs, nmb, tab, C.byref(out)), ctx)
    return out


def hydra_shard_footprint(desc, n_layers):
    out = _u64()
    _check(lib.hydra_shard_footprint(C.byref(desc), n_layers, C.byref(out)))
    return out.value


def hydra_partition(desc, mem_bound_bytes):
    """Returns (cuts, layers_per_shard): first layer of every shard of the greedy walk, and the equal shard size
    the executor can run."""
    cap = desc.n_layer + 1
    cuts = (_i32 * cap)()
    n, k = _i32(), _i32()
    _check(lib.hydra_partition(C.byref(desc), mem_bound_bytes, cuts, cap, C.byref(n), C.byref(k)))
    return [cuts[i] for i in range(n.value)], k.value


def hydra_pilot_costs(ctx, model, tokens, targets, n_shards):
    """Measured cost table (ns) of one model: forward visits of shards 0..S+1, then backward visits."""
    out = (_i64 * (2 * n_shards))()
    _check(lib.hydra_pilot_costs(ctx, model, _ptr(tokens), _ptr(targets), out), ctx)
    return [out[i] for i in range(2 * n_shards)]


def hydra_sched_destroy(s):
    return _check(lib.hydra_sched_destroy(s))


def hydra_sched_next(s):
    t = Task()
    r = _check(lib.hydra_sched_next(s, C.byref(t)))
    return None if r == 1 else (t.model, t.shard, t.phase, t.minibatch)


def hydra_sched_run(s, tokens, targets, ctx=None, trace_cap=0):
    """tokens[m], targets[m]: int32 numpy arrays [n_minibatches, B, T]. Returns the executed trace."""
    n = len(tokens)
    tk = (_vp * n)(*[_ptr(t) for t in tokens])
    tg = (_vp * n)(*[_ptr(t) for t in targets])
    trace = (Task * trace_cap)() if trace_cap else None
    done = _i64()
    _check(lib.hydra_sched_run(s, tk, tg, trace, trace_cap, C.byref(done)), ctx)
    k = min(done.value, trace_cap)
    return [(trace[i].model, trace[i].shard, trace[i].phase, trace[i].minibatch) for i in range(k)], done.value


def hydra_op_gemm(dtype, ta, tb, M, N, K, alpha, A, lda, B, ldb, bias, resid, out_f32, out_act, ldc, stream=None):
    return _check(lib.hydra_op_gemm(dtype, ta, tb, M, N, K, alpha, _ptr(A), lda, _ptr(B), ldb, _ptr(bias),
                                    _ptr(resid), _ptr(out_f32), _ptr(out_act), ldc, _stream(stream)))


def hydra_op_adam(w, m, v, g, shadow, n, lr, beta1, beta2, eps, t, stream=None):
    return _check(lib.hydra_op_adam(_ptr(w), _ptr(m), _ptr(v), _ptr(g), _ptr(shadow), n, lr, beta1, beta2, eps,
                                    t, _stream(stream)))


def hydra_op_layernorm_fwd(dtype, x, gamma, beta, y, mean, rstd, M, d, stream=None):
    return _check(lib.hydra_op_layernorm_fwd(dtype, _ptr(x), _ptr(gamma), _ptr(beta), _ptr(y), _ptr(mean),
                                             _ptr(rstd), M, d, _stream(stream)))


def hydra_op_layernorm_bwd(dy, x, mean, rstd, gamma, dres, dx, dx_bf16, dgamma, dbeta, dx_colsum, scratch, M, d,
                           stream=None):
    return _check(lib.hydra_op_layernorm_bwd(_ptr(dy), _ptr(x), _ptr(mean), _ptr(rstd), _ptr(gamma), _ptr(dres),
                                             _ptr(dx), _ptr(dx_bf16), _ptr(dgamma), _ptr(dbeta), _ptr(dx_colsum),
                                             _ptr(scratch), M, d, _stream(stream)))


def hydra_host_round_bf16(dst, src, n):
    return _check(lib.hydra_host_round_bf16(_ptr(dst), _ptr(src), n))


def hydra_op_layernorm_bwd_static(dy, x, mean, rstd, gamma, dres, dx, dx_bf16, dgamma, dbeta, dx_colsum, M, d, stream=None):
    return _check(lib.hydra_op_layernorm_bwd_static(_ptr(dy), _ptr(x), _ptr(mean), _ptr(rstd), _ptr(gamma), _ptr(dres),
                                                    _ptr(dx), _ptr(dx_bf16), _ptr(dgamma), _ptr(dbeta),
                                                    _ptr(dx_colsum), M, d, _stream(stream)))


def hydra_op_softmax_causal(dtype, S, P, n_mat, T, stream=None):
    return _check(lib.hydra_op_softmax_causal(dtype, _ptr(S), _ptr(P), n_mat, T, _stream(stream)))


def hydra_op_cross_entropy(dtype, logits, targets, row_loss, dlogits, M, V, ld, inv_n, stream=None):
    return _check(lib.hydra_op_cross_entropy(dtype, _ptr(logits), _ptr(targets), _ptr(row_loss), _ptr(dlogits), M,
                                             V, ld, inv_n, _stream(stream)))


def hydra_op_attention_fwd(qkv, o, lse, B, H, T, dh, stream=None):
    return _check(lib.hydra_op_attention_fwd(_ptr(qkv), _ptr(o), _ptr(lse), B, H, T, dh, _stream(stream)))


def hydra_op_attention_bwd(qkv, o, d_o, lse, dsum, dqkv, B, H, T, dh, stream=None):
    return _check(lib.hydra_op_attention_bwd(_ptr(qkv), _ptr(o), _ptr(d_o), _ptr(lse), _ptr(dsum), _ptr(dqkv),
                                             B, H, T, dh, _stream(stream)))
