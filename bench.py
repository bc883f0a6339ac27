#!/usr/bin/env python3
"""Throughput of spilled, shard-alternated training on one MI355X.

Headline workload (BASELINE config 5, the largest that one GPU serves): two ~6 B-parameter GPT-style decoders (28
layers, d 4096, 32 heads, MLP 16384, vocab 50400, seq 1024, batch 1; bf16 compute with fp32 master weights and
Adam state) whose 2-layer shards are alternated by the Sharded-LRTF scheduler on TWO shard buffers; all state
(145 GB) lives in host DRAM.  One step = one minibatch of every model through the whole path: promote shard,
forward visit, checkpoint, backward visit with recomputation, Adam, demote.  If the host cannot hold that state the
run falls back to config 4 (four GPT-2-XL-shaped models, 24 GB of shard buffers) and says so in config.workload.

Host state that exceeds what the driver lets a process page-lock (64 GiB on the machines this was developed on) is
kept in ordinary memory and travels through the library's page-locked staging ring.

Prints ONE JSON line.  `value` is tokens/s over all models with all inputs (weights in host memory, token batches)
prepared before the timed region.  `roofline` describes the kernel with the largest share of GPU time in a second
pass over the same work in the SAME mode (spilled, two lanes) with every launch bracketed by HIP events on its own
stream - where every byte of state crosses the host link twice per step that is the write-back copy kernel, bound
by the link; `roofline_mfma` is the matrix kernel with the largest share of the same pass.  The other BASELINE
workloads (configs 2-4) follow as objects of their own, and `cpu_baseline` times the CPU oracle on a bounded
sample of the headline workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import synth_inputs as SI  # noqa: E402

MFMA_BF16_PEAK_TFLOPS = 2500.0
HBM_PEAK_GBPS = 8000.0
PCIE_GEN5_X16_GBPS = 64.0       # per direction, theoretical
LINK_CAP_GBPS = 87.7            # both directions together, measured on this hardware (1 GB copies, SDMA in + copy kernel out:
                                # how state behind the staging area travels)
LINK_CAP_ENGINES_GBPS = 97.2    # the same with hipMemcpyAsync in both directions (how page-locked state travels): 48.6 GB/s
                                # each way in most repetitions, 41.4-49.0 over all
STAGE_BYTES = 1 << 30           # page-locked staging ring for state in ordinary memory: 2 x 8 chunks of 64 MiB

# per workload: shard buffers / byte cap as BASELINE states them (config 3 names none: three buffers per lane)
WORKLOADS = {
    "gpt6b": dict(max_slots=2, cap=0, what="2 shard buffers of 2 layers (BASELINE config 5)"),
    "gpt2xl": dict(max_slots=0, cap=24 * 10 ** 9, what="shard buffers capped at 24 GB (BASELINE config 4)"),
    "gpt2m": dict(max_slots=8, cap=0, what="8 shard buffers (two per model), every shard spilled between uses (BASELINE config 3)"),
    "gpt2s": dict(max_slots=6, cap=0, what="6 shard buffers (BASELINE config 2)"),
}


T_START = time.perf_counter()


def log(msg):
    """Progress on stderr (stdout carries the one JSON line): a run of several minutes must not look hung."""
    print(f"[bench {time.perf_counter() - T_START:6.1f}s] {msg}", file=sys.stderr, flush=True)


def mem_available_gb():
    for line in open("/proc/meminfo"):
        if line.startswith("MemAvailable:"):
            return int(line.split()[1]) * 1024 / 1e9
    return 0.0


class HostState:
    """master / m / v (and the bf16 copy) of every model of a workload.  As many of the arrays as the driver allows
    are page-locked - the second moments of all models first, then the first moments, the masters, the bf16 copies -
    and the rest is ordinary memory that the library moves through its staging area.  Weights: one seeded N(0, 0.02)
    block tiled over the master array, LayerNorm gains 1, biases 0 - cheap to produce at 6 B parameters and
    irrelevant to kernel time."""

    HEADROOM = 3 << 30      # left for the staging area, token staging and whatever else the process page-locks

    def __init__(self, cfg, n_models, R, H):
        self.cfg, self.n = cfg, n_models
        desc = H.model_desc(cfg, 1e-4)
        lay = H.hydra_model_layout(desc)
        self.n_params = lay.n_params
        self.pinned_bufs = []
        # The library's bf16 rounding of the master, which forward promotes of block shards then carry (2 instead of 4
        # bytes per parameter); kept current by host threads of the library, so nothing extra crosses the link.
        self.work_copy = WORK_COPY and cfg["dtype"] == "bf16"
        kinds = [2, 1, 0] + ([3] if self.work_copy else [])          # v, m, master, bf16 copy
        slots = {(m, k): None for k in kinds for m in range(n_models)}
        full = not PAGE_LOCK
        for k in kinds:
            for m in range(n_models):
                if full:
                    break
                try:
                    self.pinned_bufs.append(R.PinnedArray(lay.n_params, np.uint16 if k == 3 else np.float32, zero=False))
                    slots[(m, k)] = self.pinned_bufs[-1].array
                except MemoryError:
                    full = True
        if full:      # make sure the staging area will still fit
            while self.pinned_bufs:
                try:
                    R.PinnedArray(self.HEADROOM, np.uint8, zero=False).free()
                    break
                except MemoryError:
                    last = self.pinned_bufs.pop()
                    for key, a in slots.items():
                        if a is last.array:
                            slots[key] = None
                    last.free()
        self.locked = {key: a is not None for key, a in slots.items()}
        for (m, k), a in slots.items():
            if a is None:
                slots[(m, k)] = np.zeros(lay.n_params, np.uint16 if k == 3 else np.float32)
        self.arrays = [tuple(slots[(m, k)] for k in range(3)) for m in range(n_models)]
        self.work = [slots[(m, 3)] if self.work_copy else False for m in range(n_models)]
        self.pageable = not all(self.locked.values())
        lock_b = sum((2 if k == 3 else 4) for (m, k), v in self.locked.items() if v)
        self.locked_fraction = lock_b / sum((2 if k == 3 else 4) for (m, k) in self.locked)
        tensors = [H.hydra_model_tensor(desc, i) for i in range(lay.n_tensors)]
        for m in range(n_models):
            master, am, av = self.arrays[m]
            rng = np.random.default_rng(SI.model_seed(cfg, m))
            block = (rng.standard_normal(1 << 24, dtype=np.float32) * np.float32(SI.INIT_STD))
            full = master.size // block.size
            if full:
                master[: full * block.size].reshape(full, block.size)[:] = block
            master[full * block.size:] = block[: master.size - full * block.size]
            for name, off, rows, cols, _ in tensors:
                leaf = name.split(".")[-1]
                if leaf in ("ln1_g", "ln2_g", "lnf_g"):
                    master[off:off + rows * cols] = 1.0
                elif leaf.startswith("b_") or leaf in ("ln1_b", "ln2_b", "lnf_b"):
                    master[off:off + rows * cols] = 0.0
            for k, arr in ((1, am), (2, av)):
                if self.locked[(m, k)]:        # fresh ordinary memory is zero already
                    arr[:] = 0.0

    def free(self):
        self.arrays, self.work = [], []
        for b in self.pinned_bufs:
            b.free()
        self.pinned_bufs = []


PAGE_LOCK = True    # --no-page-lock: all state in ordinary memory (for comparison)
WORK_COPY = True    # --no-work-copy: forward promotes carry the fp32 master
SESSION_KW = {}     # prefetch depth / staging threads / copy workgroups from the command line (experiments)


_ARENA = [None]


def device_arena(nbytes, torch):
    """One device buffer for all contexts of the run, grown when a context needs more.  Giving the memory back after
    every context and allocating anew made the timings depend on what had run before: the context that followed
    the release of a 120 GB arena (one 6 B model fully resident) ran 17 % slower than the same context one later
    (two-model GPT-2-small workload: 112.5 against 96.1 ms per step)."""
    if _ARENA[0] is None or _ARENA[0].numel() < nbytes + 256:
        _ARENA[0] = None
        torch.cuda.empty_cache()
        _ARENA[0] = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda:0")
    return _ARENA[0]


def make_session(cfg, n_models, host, wl, flags, lanes, R, H, torch, mode="spill"):
    n_shards = n_models * (cfg["L"] // cfg["k"] + 2)
    if mode == "resident":
        slots, cap = n_shards, 0
    else:
        slots, cap = wl["max_slots"], wl["cap"]
    arena_slots = slots if slots else max(1, cap // (20 * max_shard_elems(cfg, H))) + 1
    need = R.arena_bytes_for([cfg] * n_models, arena_slots, lanes=lanes)
    sess = R.Session(need, flags=flags, max_slots=slots, shard_buffer_cap_bytes=cap, lanes=lanes,
                     stage_bytes=STAGE_BYTES if host.pageable else 0, arena=device_arena(need, torch), **SESSION_KW)
    recs = [sess.add_model(cfg, None, cfg["lrs"][m], host=host.arrays[m], pageable=host.pageable, work_copy=host.work[m])
            for m in range(n_models)]
    return sess, recs


def max_shard_elems(cfg, H):
    desc = H.model_desc(cfg, 1e-4)
    lay = H.hydra_model_layout(desc)
    return max(H.hydra_shard_range(desc, s)[1] for s in range(lay.n_shards))


def run_steps(sess, recs, cfg, n_mb, first_step, H, torch):
    n = len(recs)
    fc, bc = SI.task_costs(cfg)
    big = dict(cfg, B=cfg["B"] * cfg.get("n_micro", 1))   # a minibatch holds n_micro micro-batches of B samples
    toks = [np.stack([SI.make_batch(big, SI.batch_seed(cfg, m, first_step + i))[0] for i in range(n_mb)]) for m in range(n)]
    tgts = [np.stack([SI.make_batch(big, SI.batch_seed(cfg, m, first_step + i))[1] for i in range(n_mb)]) for m in range(n)]
    sch = H.hydra_sched_create(sess.ctx, [r["id"] for r in recs], [n_mb] * n, [list(fc) + list(bc)] * n)
    H.hydra_sync(sess.ctx)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    H.hydra_sched_run(sch, toks, tgts, sess.ctx)
    enq = time.perf_counter() - t0
    H.hydra_sync(sess.ctx)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    H.hydra_sched_destroy(sch)
    return dt, enq


def measure(cfg, n_models, host, wl, steps, warmup, R, H, torch, mode="spill", timing=False, lanes=2, extra_flags=0,
            pilot=False):
    flags = extra_flags | (H.FLAG_OVERLAP if mode == "spill" else 0) | (H.FLAG_TIMING if timing else 0)
    log(f"  {mode} pass, {steps} steps after {warmup} warm-up, {lanes} lane(s)" + (", kernels bracketed" if timing else "")
        + (f", {cfg['n_micro']} micro-batches per visit" if cfg.get("n_micro", 1) > 1 else ""))
    sess, recs = make_session(cfg, n_models, host, wl, flags, lanes, R, H, torch, mode)
    pilot_ns = None
    if pilot:   # the partitioner's pilot pass: measured cost of every shard task of model 0 (updates discarded)
        big = dict(cfg, B=cfg["B"] * cfg.get("n_micro", 1))
        tok, tgt = SI.make_batch(big, SI.batch_seed(cfg, 0, 0))
        pilot_ns = H.hydra_pilot_costs(sess.ctx, recs[0]["id"], tok, tgt, cfg["L"] // cfg["k"] + 2)
    if warmup:
        dtw, _ = run_steps(sess, recs, cfg, warmup, 0, H, torch)
        log(f"    warm-up done ({dtw:.1f} s)")
    if timing:
        H.hydra_kernel_stats_reset(sess.ctx)
    if flags & H.FLAG_OVERLAP:
        H.hydra_overlap_reset(sess.ctx)
    st0 = H.hydra_get_stats(sess.ctx)
    dt, enq = run_steps(sess, recs, cfg, steps, warmup, H, torch)
    st1 = H.hydra_get_stats(sess.ctx)
    log(f"    {steps} steps in {dt:.2f} s")
    kst = H.hydra_kernel_stats(sess.ctx) if timing else None
    ov = H.hydra_overlap_stats(sess.ctx) if flags & H.FLAG_OVERLAP else None
    losses = [H.hydra_get_loss(sess.ctx, r["id"]) for r in recs]
    sess.close()
    del sess
    torch.cuda.empty_cache()
    d = {k: st1[k] - st0[k] for k in ("bytes_h2d", "bytes_d2h", "host_promote_ms", "host_writeback_ms", "host_task_ms",
                                      "host_batch_ms")}
    return dict(seconds=dt, enqueue_seconds=enq, steps=steps, h2d=d["bytes_h2d"], d2h=d["bytes_d2h"], n_slots=st1["n_slots"],
                kernels=kst, losses=losses, pilot_ns=pilot_ns, overlap=ov, host=d)


def link_report(run, staged=False):
    s = run["seconds"]
    both = (run["h2d"] + run["d2h"]) / s / 1e9
    return {"h2d_GB_per_step": round(run["h2d"] / run["steps"] / 1e9, 3),
            "d2h_GB_per_step": round(run["d2h"] / run["steps"] / 1e9, 3),
            "h2d_GBps_over_wall": round(run["h2d"] / s / 1e9, 2), "d2h_GBps_over_wall": round(run["d2h"] / s / 1e9, 2),
            # what bounds a spilled step: both directions of the host link together carried 87.7 GB/s on this hardware
            # (each alone 57.6 / 54.7 GB/s); PCIe Gen5 x16 is 64 GB/s per direction on paper
            "both_directions_GBps_over_wall": round(both, 2),
            "both_directions_GBps_measured_cap": LINK_CAP_GBPS if staged else LINK_CAP_ENGINES_GBPS,
            "write_backs_through": "the library's copy kernel" if staged else "hipMemcpyAsync",
            "frac_of_link_cap": round(both / (LINK_CAP_GBPS if staged else LINK_CAP_ENGINES_GBPS), 3),
            "frac_of_pcie_gen5_x16_both_directions": round(both / (2 * PCIE_GEN5_X16_GBPS), 3)}


def overlap_report(run):
    """Swap / compute overlap of a run from the library's event trace.  Busy times are lengths of interval unions per
    step: a promote or write-back in flight; a shard task in flight on any lane (from its first kernel's start to its
    last kernel's end, launch gaps included: `tasks_in_flight`); and, in a pass that also brackets every kernel
    launch, a kernel executing (`kernel_busy`).  transfer_hidden_frac - the share of swap time with compute under it,
    the figure the 80 % target is judged on - is taken at kernel level where available."""
    o = run["overlap"]
    if not o or not o["n_intervals"] or o["transfer_ms"] <= 0:
        return None
    n = run["steps"]
    r = lambda x: round(x / n, 3)
    out = {"h2d_busy_ms_per_step": r(o["h2d_ms"]), "d2h_busy_ms_per_step": r(o["d2h_ms"]),
           "transfer_busy_ms_per_step": r(o["transfer_ms"]),
           "tasks_in_flight_ms_per_step": r(o["compute_ms"]),
           "tasks_in_flight_frac_of_transfer": round(o["hidden_ms"] / o["transfer_ms"], 4),
           "transfer_in_flight_frac_of_tasks": round(o["hidden_ms"] / max(o["compute_ms"], 1e-9), 4),
           "h2d_GBps_while_busy": round(o["bytes_h2d"] / max(o["h2d_ms"], 1e-9) / 1e6, 2),
           "d2h_GBps_while_busy": round(o["bytes_d2h"] / max(o["d2h_ms"], 1e-9) / 1e6, 2),
           "host_promote_ms_per_step": r(run["host"]["host_promote_ms"]),
           "host_writeback_ms_per_step": r(run["host"]["host_writeback_ms"]),
           "host_task_enqueue_ms_per_step": r(run["host"]["host_task_ms"]),
           "host_set_batch_ms_per_step": r(run["host"]["host_batch_ms"])}
    if o["kernel_ms"] > 0:
        out["kernel_busy_ms_per_step"] = r(o["kernel_ms"])
        out["transfer_hidden_frac"] = round(o["hidden_kernel_ms"] / o["transfer_ms"], 4)
        out["hidden_frac_upper_bound"] = round(min(1.0, o["kernel_ms"] / o["transfer_ms"]), 4)
    return out


def kernel_report(t):
    """Per-kernel figures of a pass with every launch bracketed by HIP events on its stream."""
    ks = sorted(t["kernels"], key=lambda k: -k["ms"])
    total_ms = sum(k["ms"] for k in ks)
    steps = t["steps"]

    def roof(k):
        avg = 1e3 * k["ms"] / k["launches"]
        if k["name"] == "copy_to_host":
            ach = k["bytes"] / (k["ms"] * 1e-3) / 1e9
            return {"bound": "link", "achieved": round(ach, 2), "peak": PCIE_GEN5_X16_GBPS, "unit": "GB/s",
                    "frac": round(ach / PCIE_GEN5_X16_GBPS, 4), "traffic": None, "kernel": k["name"],
                    "launches": k["launches"], "avg_us": round(avg, 2),
                    "peak_note": "PCIe Gen5 x16, one direction, theoretical; with promotes in flight the two directions "
                                 f"shared {LINK_CAP_GBPS} GB/s on this hardware"}
        if k["flops"] > 0:
            ach = k["flops"] / (k["ms"] * 1e-3) / 1e12
            return {"bound": "mfma", "achieved": round(ach, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(ach / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None, "kernel": k["name"],
                    "launches": k["launches"], "avg_us": round(avg, 2)}
        ach = k["bytes"] / (k["ms"] * 1e-3) / 1e9
        return {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": None, "kernel": k["name"], "launches": k["launches"],
                "avg_us": round(avg, 2)}

    gemm = [k for k in ks if k["flops"] > 0]
    out = {"roofline": roof(ks[0]),
           "kernels": [{"name": k["name"], "launches": k["launches"], "ms_per_step": round(k["ms"] / steps, 4),
                        "share": round(k["ms"] / total_ms, 4),
                        **({"TFLOPs": round(k["flops"] / (k["ms"] * 1e-3) / 1e12, 1)} if k["flops"] > 0 else
                           {"GBps": round(k["bytes"] / (k["ms"] * 1e-3) / 1e9, 1)})} for k in ks]}
    if gemm:
        tf = sum(k["flops"] for k in gemm) / (sum(k["ms"] for k in gemm) * 1e-3) / 1e12
        out["roofline_mfma"] = roof(gemm[0])
        out["gemm_aggregate"] = {"TFLOPs": round(tf, 1), "frac_of_mfma_peak": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
                                 "gemm_ms_per_step": round(sum(k["ms"] for k in gemm) / steps, 3),
                                 "kernel_ms_per_step": round(total_ms / steps, 3)}
    return out


def measured_traffic(config, kernel):
    """HBM-side bytes per launch of a kernel from the committed rocprofv3 counter summary (FETCH_SIZE and
    WRITE_SIZE runs of this script, scaled by kernels of known traffic); None when the summary has no line for it."""
    path = os.path.join(ROOT, "profiles", f"bench_{config}_hbm_counters.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) >= 3 and f[0] == "traffic_per_launch_bytes" and f[1] == kernel:
                return int(f[2])
    except OSError:
        pass
    return None


def workload_text(name, cfg, n_models, wl, host):
    return (f"{name}: {n_models} GPT-2-style decoders ({cfg['L']}L d{cfg['d']} H{cfg['H']} F{cfg['F']} V{cfg['V']}, "
            f"{host.n_params / 1e9:.3f} B parameters each), B{cfg['B']} T{cfg['T']}, {cfg['k']}-layer shards alternated by "
            f"Sharded-LRTF, {wl['what']}, bf16 MFMA + fp32 master/Adam, "
            f"{n_models * host.n_params * 12 / 1e9:.1f} GB of state in "
            + (f"host memory, {100 * host.locked_fraction:.0f} % of it page-locked (as much as the driver allows) and the rest "
               "ordinary memory whose copies are staged through a page-locked ring"
               if host.pageable else "page-locked host memory")
            + "; weights: a seeded N(0,0.02) block tiled, LayerNorm gains 1, biases 0; uniform tokens")


def bench_workload(name, steps, warmup, timing_steps, R, H, torch, n_models=0, layers=0, lanes=2, extra_flags=0,
                   micro=1):
    """One BASELINE workload as stated: spilled run (value), then the same mode with every kernel bracketed."""
    cfg = dict(SI.CONFIGS[name])
    if layers:
        cfg["L"] = layers
    if n_models:
        cfg["n_models"] = n_models
        cfg["lrs"] = (cfg["lrs"] * n_models)[:n_models]
    if micro > 1:
        cfg["n_micro"] = micro
    n = cfg["n_models"]
    wl = WORKLOADS[name]
    log(f"{name}: preparing the host state of {n} model(s)")
    host = HostState(cfg, n, R, H)
    log(f"  {n * host.n_params * 12 / 1e9:.1f} GB of state, {100 * host.locked_fraction:.0f} % of the host arrays' bytes page-locked")
    tokens = n * micro * cfg["B"] * cfg["T"]
    run = measure(cfg, n, host, wl, steps, warmup, R, H, torch, lanes=lanes, extra_flags=extra_flags)
    out = {"workload": workload_text(name, cfg, n, wl, host) + (" [depth / model count changed on the command line]" if layers or n_models else ""),
           "value": round(tokens * steps / run["seconds"], 1), "unit": "tokens/s", "steps": steps, "warmup": warmup,
           "ms_per_step": round(1e3 * run["seconds"] / steps, 3), "tokens_per_step": tokens,
           "host_enqueue_ms_per_step": round(1e3 * run["enqueue_seconds"] / steps, 3),
           "shard_buffers": run["n_slots"], "compute_lanes": lanes, "state_page_locked": not host.pageable, "host_bytes_page_locked_frac": round(host.locked_fraction, 3),
           "work_copy": host.work_copy,
           "link": link_report(run, host.pageable), "overlap": overlap_report(run),
           "final_losses": [round(x, 4) for x in run["losses"]]}
    if timing_steps:
        t = measure(cfg, n, host, wl, timing_steps, 1, R, H, torch, timing=True, lanes=lanes, extra_flags=extra_flags)
        out["kernel_pass"] = {"steps": timing_steps, "ms_per_step": round(1e3 * t["seconds"] / timing_steps, 3),
                              "overlap": overlap_report(t), **kernel_report(t)}
        # the kernels by themselves: one model, every shard resident, one lane - no second lane and no write-back
        # sharing the chip with the kernel between its two events
        q = measure(cfg, 1, host, wl, timing_steps, 1, R, H, torch, mode="resident", timing=True, lanes=1,
                    extra_flags=extra_flags)
        kq = kernel_report(q)
        out["kernels_alone"] = {"what": "one model, all shards resident, one lane: each kernel alone on the device",
                                "ms_per_step": round(1e3 * q["seconds"] / timing_steps, 3),
                                "gemm_aggregate": kq.get("gemm_aggregate"), "roofline": kq["roofline"],
                                "kernels": kq["kernels"][:12]}
    return out, cfg, host


def cpu_baseline(cfg):
    """The CPU oracle (float32 instance) on a bounded sample of the workload: whole minibatches of one model where
    that takes seconds; for the large models, steps of two depth-reduced copies (one and two block shards, same
    widths), whose difference gives the cost of a block and from it the cost of the full depth."""
    from oracle import decoder as D
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()

    def step_seconds(c, n_steps):
        W = SI.make_weights(c, SI.model_seed(c, 0))
        P = D.cast_params(W, np.float32)
        del W
        Mo, Vo = D.zeros_like_params(P), D.zeros_like_params(P)
        batches = [SI.make_batch(c, SI.batch_seed(c, 0, i)) for i in range(n_steps)]
        t0 = time.perf_counter()
        for i, (tok, tgt) in enumerate(batches):
            out = D.train_step(P, Mo, Vo, tok, tgt, c, c["lrs"][0], i + 1)
        return (time.perf_counter() - t0) / n_steps, out["loss"]

    tokens = cfg["B"] * cfg["T"]
    if SI.n_params(cfg) <= 5e8:
        n_steps = 5 if SI.n_params(cfg) <= 2e8 else 2
        log("cpu baseline: oracle on whole minibatches")
        dt, loss = step_seconds(cfg, n_steps)
        return dict(value=tokens / dt, unit="tokens/s", cores=int(threads), kind="oracle",
                    sample=f"1 model x {n_steps} minibatches ({n_steps * tokens} tokens) of the same workload, float32 "
                           f"numpy oracle, unsharded steps, {dt * n_steps:.1f} s; loss {loss:.4f}")
    k = cfg["k"]
    log("cpu baseline: oracle on depth-reduced copies")
    t1, _ = step_seconds(dict(cfg, L=k), 1)
    log(f"  depth {k}: {t1:.1f} s")
    t2, loss = step_seconds(dict(cfg, L=2 * k), 1)
    per_layer = max(t2 - t1, 1e-9) / k
    full = t1 + (cfg["L"] - k) * per_layer
    return dict(value=tokens / full, unit="tokens/s", cores=int(threads), kind="oracle",
                sample=f"float32 numpy oracle, one minibatch ({tokens} tokens) of one model at depth {k} ({t1:.1f} s) and "
                       f"{2 * k} ({t2:.1f} s), same widths, vocabulary and sequence; cost per layer {per_layer:.2f} s "
                       f"extrapolated to {cfg['L']} layers = {full:.1f} s per minibatch; loss {loss:.4f}")


def block_gemm_large_shapes(H, torch, iters=20):
    """The library's GEMM entry point on the block products of the largest configuration alone (HIP events over
    back-to-back launches, bf16 operands and result, flops = 2 M N K): context for the in-pipeline figures."""
    res = {}
    for name, (M, N, K) in {"qkv": (1024, 12288, 4096), "mlp_up": (1024, 16384, 4096), "mlp_down": (1024, 4096, 16384)}.items():
        A = torch.randn((M, K), device="cuda").to(torch.bfloat16)
        B = torch.randn((N, K), device="cuda").to(torch.bfloat16)
        C = torch.empty((M, N), device="cuda", dtype=torch.bfloat16)
        call = lambda: H.hydra_op_gemm(1, 0, 0, M, N, K, 1.0, A, K, B, K, None, None, None, C, N)
        for _ in range(3):
            call()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(iters):
            call()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / iters
        tf = 2.0 * M * N * K / us / 1e6
        res[name] = {"MxNxK": f"{M}x{N}x{K}", "us": round(us, 1), "TFLOPs": round(tf, 1),
                     "frac_of_mfma_peak": round(tf / MFMA_BF16_PEAK_TFLOPS, 4)}
    return res


def gpt2s_extras(cfg, host, R, H, torch, steps):
    """Config 2 beyond the stated run: everything resident (the compute-bound figure), pilot-pass costs, the
    partitioner's footprints, and several micro-batches per shard visit (same state traffic, more tokens)."""
    wl = WORKLOADS["gpt2s"]
    n = cfg["n_models"]
    tokens = n * cfg["B"] * cfg["T"]
    out = {}
    o = measure(cfg, n, host, wl, steps, 2, R, H, torch, mode="resident", pilot=True)
    n_sh = cfg["L"] // cfg["k"] + 2
    out["pilot_costs_us"] = {"forward": [round(x / 1e3, 1) for x in o["pilot_ns"][:n_sh]],
                             "backward_with_adam": [round(x / 1e3, 1) for x in o["pilot_ns"][n_sh:]],
                             "shards": "EMBED, block shards 1..S, HEAD; model 0, each task alone on the device"}
    fp = [H.hydra_shard_footprint(H.model_desc(cfg, 1e-4), k) for k in range(0, cfg["L"] + 1)]
    out["partitioner"] = {"footprint_MB_by_layers_in_shard": [round(x / 1e6, 1) for x in fp[1:]],
                          "embed_head_MB": round(fp[0] / 1e6, 1),
                          "cuts_at_bound_of_2_layer_shard": H.hydra_partition(H.model_desc(cfg, 1e-4), max(fp[2], fp[0]))[0]}
    out["resident"] = {"value": round(tokens * steps / o["seconds"], 1), "unit": "tokens/s",
                       "ms_per_step": round(1e3 * o["seconds"] / steps, 3),
                       "host_enqueue_ms_per_step": round(1e3 * o["enqueue_seconds"] / steps, 3), "shard_buffers": o["n_slots"]}
    steps_m = max(2, steps // 2)
    for nm in (4, 8):
        # plain launches: replaying visits as graphs saved host time while the host was the bottleneck of these runs;
        # it no longer is, and the gate that keeps the library's threads out of the runtime during a capture costs more
        # (172 k against 163 k tokens/s with four micro-batches, 334 k against 313 k with eight)
        mc = dict(cfg, n_micro=nm)
        o = measure(mc, n, host, wl, steps_m, 2, R, H, torch)
        tt = measure(mc, n, host, wl, 2, 1, R, H, torch, timing=True)
        out[f"spill_micro{nm}"] = {"value": round(tokens * nm * steps_m / o["seconds"], 1), "unit": "tokens/s",
                                   "ms_per_step": round(1e3 * o["seconds"] / steps_m, 3), "tokens_per_step": tokens * nm,
                                   "hip_graphs": False, "link": link_report(o, host.pageable), "overlap": overlap_report(o),
                                   "kernel_pass_overlap": overlap_report(tt)}
    return out


def main():
    global WORK_COPY, PAGE_LOCK
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="auto", help="headline workload: gpt6b (default when the host holds its 145 GB "
                    "of state), gpt2xl, gpt2m or gpt2s")
    ap.add_argument("--only", action="store_true", help="measure the headline workload only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-pass", action="store_true", help="skip the pass that brackets every kernel launch")
    ap.add_argument("--large-gemm-only", action="store_true",
                    help="only time the block products of the largest configuration (for counter runs) and print them")
    ap.add_argument("--lanes", type=int, default=2, help="compute lanes (streams); models are spread over them")
    ap.add_argument("--layers", type=int, default=0, help="cut the model depth of the headline workload (reported)")
    ap.add_argument("--models", type=int, default=0, help="number of models of the headline workload (reported)")
    ap.add_argument("--micro", type=int, default=1, help="micro-batches of B samples per shard visit (1 = as stated)")
    ap.add_argument("--graphs", action="store_true", help="replay block-shard visits as HIP graphs")
    ap.add_argument("--ckpt-spill", action="store_true", help="boundary activations travel through host DRAM too")
    ap.add_argument("--d2h-memcpy", action="store_true", help="every write-back through hipMemcpyAsync (default: page-locked state only)")
    ap.add_argument("--d2h-kernel", action="store_true", help="every write-back through the library's copy kernel (default: staged state only)")
    ap.add_argument("--no-page-lock", action="store_true", help="keep all model state in ordinary host memory")
    ap.add_argument("--no-work-copy", action="store_true",
                    help="no bf16 copy of the master on the host: forward promotes carry the fp32 master")
    ap.add_argument("--prefetch-depth", type=int, default=0, help="tasks ahead that shards are promoted for (0 = as far as buffers allow)")
    ap.add_argument("--stage-threads", type=int, default=0, help="host threads per direction of the staging tier (0 = 5)")
    ap.add_argument("--copy-blocks", type=int, default=0, help="workgroups of the write-back copy kernel (0 = by tokens per visit)")
    ap.add_argument("--slots", type=int, default=0, help="shard buffers of the headline workload (0 = as BASELINE states)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the method shards over host DRAM, not over GPUs); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2110_08633_amd import hydra as H, runtime as R
    assert torch.cuda.is_available(), "no GPU visible"
    if args.large_gemm_only:
        print(json.dumps({"block_gemm_large_shapes": block_gemm_large_shapes(H, torch)}))
        return
    flags = (H.FLAG_GRAPHS if args.graphs else 0) | (H.FLAG_CKPT_SPILL if args.ckpt_spill else 0) | \
            (H.FLAG_D2H_MEMCPY if args.d2h_memcpy else 0) | (H.FLAG_D2H_KERNEL if args.d2h_kernel else 0)
    WORK_COPY = not args.no_work_copy
    PAGE_LOCK = not args.no_page_lock
    SESSION_KW.update(prefetch_depth=args.prefetch_depth, stage_threads=args.stage_threads, copy_blocks=args.copy_blocks)
    avail = mem_available_gb()
    name = args.config
    fallback = None
    if name == "auto":
        # config 5 keeps 145 GB of state and 24 GB of bf16 copies in host DRAM (plus what the process itself needs)
        name = "gpt6b" if avail >= 200 else "gpt2xl"
        if name != "gpt6b":
            fallback = f"host has {avail:.0f} GB available: config 5's 170 GB of state do not fit, config 4 measured instead"
    if args.slots:
        WORKLOADS[name] = dict(WORKLOADS[name], max_slots=args.slots, cap=0, what=f"{args.slots} shard buffers [command line]")
    main_out, cfg, host = bench_workload(name, args.steps, args.warmup, 0 if args.no_kernel_pass else 2, R, H, torch,
                                         n_models=args.models, layers=args.layers, lanes=args.lanes, extra_flags=flags,
                                         micro=args.micro)
    out = {"metric": "training tokens/sec (all models, 1 MI355X)", "value": main_out["value"], "unit": "tokens/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_out["ms_per_step"],
           "host_enqueue_ms_per_step": main_out["host_enqueue_ms_per_step"], "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": main_out["workload"], "mode": "spill", "shard_buffers": main_out["shard_buffers"],
                      "compute_lanes": args.lanes, "hip_graphs": args.graphs, "checkpoints_through_host": args.ckpt_spill,
                      "micro_batches_per_visit": args.micro, "tokens_per_step": main_out["tokens_per_step"],
                      "host_memory_available_GB": round(avail, 1), "state_page_locked": main_out["state_page_locked"],
                      "host_bytes_page_locked_frac": main_out["host_bytes_page_locked_frac"],
                      "bf16_host_copy_for_forward_promotes": main_out["work_copy"]},
           "link": main_out["link"], "overlap": main_out["overlap"], "final_losses": main_out["final_losses"]}
    if fallback:
        out["config"]["fallback"] = fallback
    if "kernel_pass" in main_out:
        kp = main_out["kernel_pass"]
        out["roofline"] = kp["roofline"]
        out["roofline"]["traffic"] = measured_traffic(name, kp["roofline"]["kernel"])
        if "roofline_mfma" in kp:
            out["roofline_mfma"] = kp["roofline_mfma"]
            out["roofline_mfma"]["traffic"] = measured_traffic(name, kp["roofline_mfma"]["kernel"])
            out["gemm_aggregate"] = kp["gemm_aggregate"]
        out["kernels_alone"] = main_out["kernels_alone"]
        out["kernel_pass"] = {"what": "the same steps in the same mode with every kernel launch bracketed by HIP events",
                              "steps": kp["steps"], "ms_per_step": kp["ms_per_step"], "overlap": kp["overlap"]}
        out["kernels"] = kp["kernels"]
    cpu_cfg = cfg
    host.free()
    del host
    if not args.only:
        for other, (st, wu) in {"gpt2s": (16, 2), "gpt2m": (5, 1), "gpt2xl": (3, 1)}.items():
            if other == name:
                continue
            o, ocfg, ohost = bench_workload(other, st, wu, 0 if args.no_kernel_pass else 2, R, H, torch, lanes=args.lanes)
            if "kernel_pass" in o:
                o["kernel_pass"]["kernels"] = o["kernel_pass"]["kernels"][:8]
            if other == "gpt2s":
                o.update(gpt2s_extras(ocfg, ohost, R, H, torch, st))
            ohost.free()
            del ohost
            out[other] = o
        out["block_gemm_large_shapes"] = block_gemm_large_shapes(H, torch)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cpu_cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
