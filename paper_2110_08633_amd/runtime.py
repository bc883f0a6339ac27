"""Plumbing around the C ABI: device arena, pinned host state, streams.

torch is used only to allocate memory and create streams; every computation
happens inside libhydra.so.  With dry_run=True no GPU is touched (host-only
state machine tests).
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import hydra as H

_hip = None


def _hip_runtime():
    """The HIP runtime already loaded into this process (torch's), so that host memory page-locked here is known to
    the runtime the library and torch use."""
    global _hip
    if _hip is None:
        path = None
        with open("/proc/self/maps") as f:
            for line in f:
                if "libamdhip64" in line:
                    path = line.split()[-1]
                    break
        if path is None:
            raise RuntimeError("no HIP runtime is loaded in this process")
        _hip = C.CDLL(path)
        _hip.hipHostMalloc.argtypes = [C.POINTER(C.c_void_p), C.c_size_t, C.c_uint]
        _hip.hipHostFree.argtypes = [C.c_void_p]
    return _hip


class PinnedArray:
    """Page-locked host memory from hipHostMalloc, viewed as a numpy array; released by free() (torch's pinned
    allocator rounds sizes up to powers of two and keeps what it is given back, which does not suit arrays of tens
    of gigabytes).  Fresh pages read as zero; zero=True clears them regardless."""

    def __init__(self, n, dtype=np.float32, zero=True):
        self.nbytes = max(int(n) * np.dtype(dtype).itemsize, 16)
        p = C.c_void_p()
        e = _hip_runtime().hipHostMalloc(C.byref(p), self.nbytes, 0)
        if e != 0 or not p.value:
            _hip_runtime().hipGetLastError()      # the failed call's error must not surface at the next HIP call
            raise MemoryError(f"hipHostMalloc of {self.nbytes} bytes failed (HIP error {e})")
        self.ptr = p.value
        if zero:
            C.memset(self.ptr, 0, self.nbytes)
        self.array = np.frombuffer((C.c_char * self.nbytes).from_address(self.ptr), dtype=dtype, count=int(n))

    def free(self):
        if self.ptr:
            self.array = None
            _hip_runtime().hipHostFree(self.ptr)
            self.ptr = None


_STREAMS = {}


def independent_streams(n):
    """n streams (default priority) of which as many as possible do not hold each other up.

    HIP multiplexes a process's streams onto a few hardware queues (four by default), work of streams that share one
    runs in order, and which streams share is not round-robin: of torch's pooled streams 2 and 3 shared a queue on
    the machines this was developed on.  The swap engine needs its promote stream, its write-back stream and the
    compute lanes to really run side by side (with two of them on one queue the two-model GPT-2-small workload took
    108-112 instead of 96 ms per step), so candidates are tried pair by pair: a spin kernel of about a millisecond on
    one, a tiny kernel on the other; streams whose tiny kernel had to wait for the spin share a queue.  Chosen once
    per process and count."""
    if n in _STREAMS:
        return _STREAMS[n]
    import torch
    x = torch.zeros(64, device="cuda:0")

    def held_up(a, b):
        torch.cuda.synchronize()
        ea, eb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(a):
            torch.cuda._sleep(2_500_000)
            ea.record(a)
        with torch.cuda.stream(b):
            x.add_(1.0)
            eb.record(b)
        torch.cuda.synchronize()
        return eb.elapsed_time(ea) < 0.25      # b's kernel ended less than 0.25 ms before a's spin (or after it)

    chosen, rest = [], []
    try:
        warm = torch.cuda.Stream()
        held_up(warm, warm)                    # first use of the spin kernel and of the events
        rest.append(warm)
        for _ in range(24):
            if len(chosen) >= n:
                break
            c = torch.cuda.Stream()
            if all(not held_up(k, c) for k in chosen):
                chosen.append(c)
            else:
                rest.append(c)
    except Exception:                          # no spin kernel in this torch build: take streams as they come
        pass
    while len(chosen) < n:                     # more streams than hardware queues (or no test): the others share
        chosen.append(rest.pop() if rest else torch.cuda.Stream())
    _STREAMS[n] = chosen
    return chosen


class Session:
    """One hydra context with its arena, three streams and registered models."""

    def __init__(self, arena_bytes, flags=0, shard_buffer_cap_bytes=0, max_slots=0, dry_run=False, lanes=1,
                 copy_blocks=0, prefetch_depth=0, stage_bytes=0, stage_threads=0, arena=None):
        """stage_bytes > 0: a page-locked staging area of that size is handed to the library, and models may be added
        with pageable=True (master / m / v in ordinary memory, for state beyond what can be page-locked).
        arena: a uint8 device tensor of at least arena_bytes + 256 to use instead of allocating one (a process that
        opens one context after another can keep its device memory that way)."""
        self.dry = dry_run
        self.models = []      # dicts: desc, cfg, master, m, v, ckpt, id, names
        self._pinned = []
        if dry_run:
            flags |= H.FLAG_DRY_RUN
            self.arena = None
            self.streams = (None, None, None)
            self.lane_streams = []
            arena_ptr = 256
        else:
            import torch
            self.torch = torch
            if arena is not None and arena.numel() < arena_bytes + 256:
                raise ValueError("arena tensor too small")
            self.arena = arena if arena is not None else torch.empty(arena_bytes + 256, dtype=torch.uint8, device="cuda:0")
            arena_ptr = (self.arena.data_ptr() + 255) // 256 * 256
            # promote, write-back and the first lanes on hardware queues of their own (compute, h2d, d2h, lanes 1..)
            pool = independent_streams(2 + lanes)
            self.streams = (pool[2], pool[0], pool[1])
            self.lane_streams = pool[3:]
        self.stage = None
        if stage_bytes and not dry_run:
            self.stage = PinnedArray(stage_bytes + 256, np.uint8, zero=False)
            self._pinned.append(self.stage)
        stage_ptr = (self.stage.ptr + 255) // 256 * 256 if self.stage else None
        self.ctx = H.hydra_init(arena_ptr, arena_bytes, *self.streams, flags=flags, stage=stage_ptr,
                                stage_bytes=stage_bytes if self.stage else 0, stage_threads=stage_threads,
                                shard_buffer_cap_bytes=shard_buffer_cap_bytes, max_slots=max_slots,
                                compute_lanes=lanes, lane_streams=self.lane_streams, copy_blocks=copy_blocks,
                                prefetch_depth=prefetch_depth)
        self.flags = flags

    def _host(self, n, dtype=np.float32, pageable=False):
        if self.dry or pageable:
            return np.zeros(n, dtype)
        buf = PinnedArray(n, dtype)
        self._pinned.append(buf)
        return buf.array

    def add_model(self, cfg, weights, lr, dtype=None, pageable=False, host=None, work_copy=False):
        """weights: dict name -> float32 array (names as given by hydra_model_tensor), or None to leave the master
        array as it is.  pageable: the model's state arrays are ordinary host memory (needs a session with a staging
        area).  host: (master, m, v) arrays to use instead of allocating (they stay the caller's).  work_copy: also
        give the library a bf16 array of the model's size, page-locked or not as the state is (forward promotes of
        block shards then carry 2 instead of 4 bytes per parameter); True allocates it, an array is used as it is."""
        desc = H.model_desc(cfg, lr, dtype)
        lay = H.hydra_model_layout(desc)
        master, m, v = host if host is not None else (self._host(lay.n_params, pageable=pageable) for _ in range(3))
        tensors = {}
        for i in range(lay.n_tensors):
            name, off, rows, cols, shard = H.hydra_model_tensor(desc, i)
            tensors[name] = (off, rows, cols, shard)
            if weights is not None:
                master[off:off + rows * cols] = np.asarray(weights[name], np.float32).reshape(-1)
        ckpt = None
        if self.flags & H.FLAG_CKPT_SPILL:
            ckpt = self._host((lay.n_block_shards + 1) * cfg.get("n_micro", 1) * cfg["B"] * cfg["T"] * cfg["d"])
        stage = self._host(4 * cfg.get("n_micro", 1) * cfg["B"] * cfg["T"], np.int32)
        if isinstance(work_copy, np.ndarray):
            work = work_copy                      # the caller's array
        else:
            work = self._host(lay.n_params, np.uint16, pageable=pageable) if work_copy else None
        mid = H.hydra_register_model(self.ctx, desc, master, m, v, ckpt, stage, work)
        rec = dict(id=mid, desc=desc, cfg=cfg, layout=lay, master=master, m=m, v=v, ckpt=ckpt, stage=stage, tensors=tensors,
                   S=lay.n_block_shards, work=work)
        self.models.append(rec)
        return rec

    def unpack(self, rec, flat):
        """dict name -> array view of a flat array in canonical layout."""
        return {n: flat[o:o + r * c].reshape((r, c) if c > 1 else (r,)) for n, (o, r, c, _) in rec["tensors"].items()}

    def read_shard(self, rec, shard, which):
        off, cnt = H.hydra_shard_range(rec["desc"], shard)
        out = np.empty(cnt, np.float32)
        H.hydra_read_device(self.ctx, rec["id"], shard, which, out)
        return out

    def read_logits(self, rec):
        """Logits of the last micro-batch of the model's last HEAD forward."""
        cfg = rec["cfg"]
        out = np.empty((cfg["B"] * cfg["T"], cfg["V"]), np.float32)
        H.hydra_read_device(self.ctx, rec["id"], 0, H.RD_LOGITS, out)
        return out

    def read_act(self, rec, shard, which):
        cfg = rec["cfg"]
        out = np.empty((cfg.get("n_micro", 1) * cfg["B"] * cfg["T"], cfg["d"]), np.float32)
        H.hydra_read_device(self.ctx, rec["id"], shard, which, out)
        return out

    def train_step_manual(self, rec, tokens, targets, collect=True, spill=True):
        """One minibatch of one model through the low-level calls, shard by
        shard.  Returns logits, loss and a dict of gradients (read back before
        each shard's Adam step) when collect is set."""
        ctx, mid, S = self.ctx, rec["id"], rec["S"]
        H.hydra_set_batch(ctx, mid, np.ascontiguousarray(tokens, np.int32), np.ascontiguousarray(targets, np.int32))
        for s in range(S + 2):
            H.hydra_shard_load_async(ctx, mid, s, H.LOAD_PARAMS)
            H.hydra_shard_forward(ctx, mid, s)
            if spill and s != S + 1:
                H.hydra_shard_spill(ctx, mid, s, H.SPILL_EVICT)
        out = {}
        if collect:
            out["logits"] = self.read_logits(rec)
        out["loss"] = H.hydra_get_loss(ctx, mid)
        gflat = np.zeros(rec["layout"].n_params, np.float32)
        for s in range(S + 1, -1, -1):
            H.hydra_shard_load_async(ctx, mid, s, H.LOAD_PARAMS | H.LOAD_OPT)
            H.hydra_shard_backward(ctx, mid, s)
            if collect:
                off, cnt = H.hydra_shard_range(rec["desc"], s)
                gflat[off:off + cnt] = self.read_shard(rec, s, H.RD_GRADS)
            H.hydra_shard_adam_step(ctx, mid, s)
            if spill:
                H.hydra_shard_spill(ctx, mid, s, H.SPILL_WRITEBACK | H.SPILL_EVICT)
        if collect:
            out["grads"] = self.unpack(rec, gflat)
        return out

    def flush(self):
        """Write every resident shard's changed state back to the host arrays."""
        for rec in self.models:
            for s in range(rec["S"] + 2):
                try:
                    H.hydra_shard_spill(self.ctx, rec["id"], s, H.SPILL_WRITEBACK)
                except H.HydraError as e:
                    if e.code != H.E_STATE:
                        raise
        H.hydra_sync(self.ctx)

    def close(self):
        """Destroys the context and releases the page-locked arrays: views of them (rec["master"] ...) die here."""
        if self.ctx is not None:
            H.hydra_destroy(self.ctx)
            self.ctx = None
        for rec in self.models:
            for k in ("master", "m", "v", "ckpt", "stage", "work"):
                rec[k] = None
        for buf in self._pinned:
            buf.free()
        self._pinned = []


def arena_bytes_for(cfgs, n_slots, ckpt_spill=False, lanes=1):
    """Generous arena size for a list of model configs and a number of shard buffers."""
    total, ws, max_shard = 0, 0, 0
    for c in cfgs:
        M, d, F, V, T, B, k = c["B"] * c["T"], c["d"], c["F"], c["V"], c["T"], c["B"], c["k"]
        S = c["L"] // k
        act = M * d * 4
        vpad = (V + 63) // 64 * 64
        nm = c.get("n_micro", 1)
        total += nm * ((2 if ckpt_spill else S + 1) * act + 2 * act + M * vpad * 4 + 64 * M) + (1 << 16)
        if c.get("tie"):
            total += V * d * 4 + 256
        layer = 5 * act + 3 * M * d * 4 + M * 3 * d * 4 + B * c["H"] * T * T * 4 + 2 * M * F * 4
        scratch = 2 * B * c["H"] * T * T * 4 + 4 * act + M * F * 4 + M * 3 * d * 4 + 4 * act
        # activation gradients kept per block of a backward visit, and the partial column sums behind its
        # bias / LayerNorm gradients
        grads = 6 * act + M * F * 4 + M * 3 * d * 4 + (M // 8 + 1) * 6 * d * 4 + (M // 128 + 1) * (F + 3 * d) * 4 + 4096
        ws = max(ws, k * (layer + act + grads) + scratch + 2 * act + (1 << 20), M * vpad * 4 + 4 * act + (1 << 20))
        blk = 12 * d * d + 13 * d if F == 4 * d else 4 * d * d + 2 * d * F + 9 * d + F
        max_shard = max(max_shard, V * d + T * d, k * blk, 2 * d + d * V)
    return int(total + lanes * ws + n_slots * (max_shard * 20 + 4096) + (64 << 20))
