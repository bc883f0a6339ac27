#!/usr/bin/env python3
"""Throughput of spilled, shard-alternated training on one MI355X.

Workload (BASELINE config 2): two GPT-2-small-shaped models (12 layers, d 768,
12 heads, MLP 3072, vocab 50257, seq 512, batch 4; bf16 compute with fp32
master weights; lr 1e-4 / 3e-5) whose 2-layer shards are alternated by the
Sharded-LRTF scheduler.  One step = one minibatch of every model through the
whole path: promote shard, forward visit, checkpoint, backward visit with
recomputation, Adam, demote.

Default mode "spill": six shard buffers (per compute lane one computing, one filling, one draining), so every shard's state streams in
from pinned host DRAM before each visit and the updated state streams back.
Mode "resident": as many buffers as shards (state crosses the link once).

Prints ONE JSON line.  `value` is tokens/s over all models with all inputs
(weights in pinned host memory, token batches) prepared before the timed
region.  `roofline` describes the kernel with the largest share of GPU time,
timed with HIP events on its own stream in a second pass over the same work.
`cpu_baseline` times the CPU oracle on a bounded sample of the same workload.
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


SPILL_SLOTS = 4
TRACE_OVERLAP = True
EXTRA_FLAGS = 0
LINK_CAP_GBPS = 87.7
LANES = 2


def make_session(cfg, n_models, mode, timing, R, H):
    n_shards = n_models * (cfg["L"] // cfg["k"] + 2)
    slots = SPILL_SLOTS if mode == "spill" else n_shards
    # event pairs around promotes, write-backs and tasks (a few hundred per step) give the overlap figures
    flags = (H.FLAG_TIMING if timing else (H.FLAG_OVERLAP if TRACE_OVERLAP and mode == "spill" else 0)) | EXTRA_FLAGS
    lanes = 1 if timing else LANES      # per-kernel timing wants kernels one at a time
    sess = R.Session(R.arena_bytes_for([cfg] * n_models, slots, lanes=lanes), flags=flags, max_slots=slots, lanes=lanes)
    recs = []
    for m in range(n_models):
        W = SI.make_weights(cfg, SI.model_seed(cfg, m))
        recs.append(sess.add_model(cfg, W, cfg["lrs"][m]))
        del W
    return sess, recs


def flags_have_overlap(sess, H):
    return bool(sess.flags & H.FLAG_OVERLAP)


def run_steps(sess, recs, cfg, n_mb, first_step, H, torch):
    n = len(recs)
    fc, bc = SI.task_costs(cfg)
    big = dict(cfg, B=cfg["B"] * cfg.get("n_micro", 1))   # a minibatch holds n_micro micro-batches of B samples
    toks = [np.stack([SI.make_batch(big, SI.batch_seed(cfg, m, first_step + i))[0] for i in range(n_mb)]) for m in range(n)]
    tgts = [np.stack([SI.make_batch(big, SI.batch_seed(cfg, m, first_step + i))[1] for i in range(n_mb)]) for m in range(n)]
    sch = H.hydra_sched_create(sess.ctx, [r["id"] for r in recs], [n_mb] * n, [list(fc) + list(bc)] * n)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    H.hydra_sched_run(sch, toks, tgts, sess.ctx)
    run_steps.enqueue_s = time.perf_counter() - t0
    H.hydra_sync(sess.ctx)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    H.hydra_sched_destroy(sch)
    return dt


def measure(cfg, n_models, mode, steps, warmup, timing, R, H, torch, pilot=False):
    sess, recs = make_session(cfg, n_models, mode, timing, R, H)
    pilot_ns = None
    if pilot:   # the partitioner's pilot pass: measured cost of every shard task of model 0 (updates discarded)
        big = dict(cfg, B=cfg["B"] * cfg.get("n_micro", 1))
        tok, tgt = SI.make_batch(big, SI.batch_seed(cfg, 0, 0))
        pilot_ns = H.hydra_pilot_costs(sess.ctx, recs[0]["id"], tok, tgt, cfg["L"] // cfg["k"] + 2)
    if warmup:
        run_steps(sess, recs, cfg, warmup, 0, H, torch)
    if timing:
        H.hydra_kernel_stats_reset(sess.ctx)
    elif flags_have_overlap(sess, H):
        H.hydra_overlap_reset(sess.ctx)
    st0 = H.hydra_get_stats(sess.ctx)
    dt = run_steps(sess, recs, cfg, steps, warmup, H, torch)
    st1 = H.hydra_get_stats(sess.ctx)
    kst = H.hydra_kernel_stats(sess.ctx) if timing else None
    ov = H.hydra_overlap_stats(sess.ctx) if flags_have_overlap(sess, H) else None
    losses = [H.hydra_get_loss(sess.ctx, r["id"]) for r in recs]
    sess.close()
    del sess
    torch.cuda.empty_cache()
    return dict(seconds=dt, enqueue_seconds=run_steps.enqueue_s, h2d=st1["bytes_h2d"] - st0["bytes_h2d"], d2h=st1["bytes_d2h"] - st0["bytes_d2h"],
                n_slots=st1["n_slots"], kernels=kst, losses=losses, pilot_ns=pilot_ns, overlap=ov,
                host_promote_ms=st1["host_promote_ms"] - st0["host_promote_ms"],
                host_writeback_ms=st1["host_writeback_ms"] - st0["host_writeback_ms"],
                host_task_ms=st1["host_task_ms"] - st0["host_task_ms"],
                host_batch_ms=st1["host_batch_ms"] - st0["host_batch_ms"])


def overlap_report(run, steps):
    """Swap / compute overlap of a run from the library's event trace: busy times are lengths of interval unions
    (a shard task running on any lane; a promote or a write-back in flight), per step."""
    o = run["overlap"]
    if not o or not o["n_intervals"] or o["transfer_ms"] <= 0:
        return None
    r = lambda x: round(x / steps, 3)
    return {"compute_busy_ms_per_step": r(o["compute_ms"]), "h2d_busy_ms_per_step": r(o["h2d_ms"]),
            "d2h_busy_ms_per_step": r(o["d2h_ms"]), "transfer_busy_ms_per_step": r(o["transfer_ms"]),
            "transfer_hidden_frac": round(o["hidden_ms"] / o["transfer_ms"], 4),
            "hidden_frac_upper_bound": round(min(1.0, o["compute_ms"] / o["transfer_ms"]), 4),
            "compute_with_transfer_in_flight_frac": round(o["hidden_ms"] / max(o["compute_ms"], 1e-9), 4),
            "h2d_GBps_while_busy": round(o["bytes_h2d"] / max(o["h2d_ms"], 1e-9) / 1e6, 2),
            "d2h_GBps_while_busy": round(o["bytes_d2h"] / max(o["d2h_ms"], 1e-9) / 1e6, 2),
            "host_promote_ms_per_step": r(run["host_promote_ms"]), "host_writeback_ms_per_step": r(run["host_writeback_ms"]),
            "host_task_enqueue_ms_per_step": r(run["host_task_ms"]), "host_set_batch_ms_per_step": r(run["host_batch_ms"])}


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


def cpu_baseline(cfg):
    """The CPU oracle (float32 instance) on one model-minibatch of the same workload."""
    from oracle import decoder as D
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()
    W = SI.make_weights(cfg, SI.model_seed(cfg, 0))
    P = D.cast_params(W, np.float32)
    Mo, Vo = D.zeros_like_params(P), D.zeros_like_params(P)
    n_steps = 5
    batches = [SI.make_batch(cfg, SI.batch_seed(cfg, 0, i)) for i in range(n_steps)]
    t0 = time.perf_counter()
    for i, (tok, tgt) in enumerate(batches):
        out = D.train_step(P, Mo, Vo, tok, tgt, cfg, cfg["lrs"][0], i + 1)
    dt = time.perf_counter() - t0
    return dict(value=n_steps * cfg["B"] * cfg["T"] / dt, unit="tokens/s", cores=int(threads), kind="oracle",
                sample=f"1 model x {n_steps} minibatches ({n_steps * cfg['B'] * cfg['T']} tokens) of the same workload, "
                       f"float32 numpy oracle, unsharded steps, {dt:.1f} s; loss {out['loss']:.4f}")


def block_gemm_large_shapes(H, torch, iters=20):
    """Context beside the workload's own figures: the library's GEMM entry point on the block products of the
    largest configuration (28 layers, d 4096, F 16384, 1024 tokens per visit), where a product fills the chip:
    HIP events over back-to-back launches, bf16 operands, bf16 result, flops = 2 M N K."""
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=16)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--mode", choices=["spill", "resident"], default="spill")
    ap.add_argument("--config", default="gpt2s")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the second mode and the timing pass")
    ap.add_argument("--large-gemm-only", action="store_true",
                    help="only time the block products of the largest configuration (for counter runs) and print them")
    ap.add_argument("--slots", type=int, default=6, help="shard buffers in spill mode (three per compute lane)")
    ap.add_argument("--d2h-memcpy", action="store_true", help="demote with hipMemcpyAsync instead of the copy kernel")
    ap.add_argument("--lanes", type=int, default=2, help="compute lanes (streams); models are spread over them")
    ap.add_argument("--graphs", action="store_true",
                    help="replay block-shard visits as HIP graphs (halves the host's enqueue time; the device is the "
                         "bottleneck at this workload, so the throughput does not move)")
    ap.add_argument("--ckpt-spill", action="store_true",
                    help="boundary activations travel through host DRAM between visits (HYDRA_FLAG_CKPT_SPILL)")
    ap.add_argument("--layers", type=int, default=0, help="cut the model depth (other configs than the default: a "
                    "depth-reduced copy with full widths; reported in config)")
    ap.add_argument("--models", type=int, default=0, help="number of models (default: the config's)")
    ap.add_argument("--no-overlap-trace", action="store_true",
                    help="spill mode: do not record the event pairs behind the 'overlap' figures")
    ap.add_argument("--micro", type=int, default=1,
                    help="micro-batches of B samples per shard visit (1 = the workload as BASELINE states it)")
    ap.add_argument("--extra-micro", type=int, default=4,
                    help="also report spill-mode throughput with this many micro-batches per visit (0 = skip)")
    args = ap.parse_args()
    global SPILL_SLOTS, EXTRA_FLAGS, LANES, TRACE_OVERLAP
    TRACE_OVERLAP = not args.no_overlap_trace
    SPILL_SLOTS = args.slots
    LANES = args.lanes
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
    if args.d2h_memcpy:
        EXTRA_FLAGS |= H.FLAG_D2H_MEMCPY
    if args.graphs:
        EXTRA_FLAGS |= H.FLAG_GRAPHS
    if args.ckpt_spill:
        EXTRA_FLAGS |= H.FLAG_CKPT_SPILL
    cfg = dict(SI.CONFIGS[args.config])
    if args.micro > 1:
        cfg["n_micro"] = args.micro
    if args.layers:
        cfg["L"] = args.layers
    if args.models:
        cfg["n_models"] = args.models
        cfg["lrs"] = (cfg["lrs"] * args.models)[:args.models]
    n_models = cfg["n_models"]
    tokens_per_step = n_models * args.micro * cfg["B"] * cfg["T"]

    main_run = measure(cfg, n_models, args.mode, args.steps, args.warmup, False, R, H, torch)
    value = tokens_per_step * args.steps / main_run["seconds"]
    out = {
        "metric": "training tokens/sec (all models, 1 MI355X)", "value": round(value, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(1e3 * main_run["seconds"] / args.steps, 3),
        "host_enqueue_ms_per_step": round(1e3 * main_run["enqueue_seconds"] / args.steps, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.config}: {n_models} GPT-2-shaped models ({cfg['L']}L d{cfg['d']} H{cfg['H']} "
                               f"F{cfg['F']} V{cfg['V']}), B{cfg['B']} T{cfg['T']}, {cfg['k']}-layer shards alternated by "
                               "Sharded-LRTF, bf16 MFMA + fp32 master/Adam, seeded N(0,0.02) weights, uniform tokens"
                               + (" [depth / model count reduced on the command line]" if args.layers or args.models else ""),
                   "mode": args.mode, "shard_buffers": main_run["n_slots"], "compute_lanes": args.lanes, "hip_graphs": args.graphs, "checkpoints_through_host": args.ckpt_spill,
                   "micro_batches_per_visit": args.micro, "tokens_per_step": tokens_per_step},
        "link": {"h2d_GB_per_step": round(main_run["h2d"] / args.steps / 1e9, 3),
                 "d2h_GB_per_step": round(main_run["d2h"] / args.steps / 1e9, 3),
                 "h2d_GBps_over_wall": round(main_run["h2d"] / main_run["seconds"] / 1e9, 2),
                 "d2h_GBps_over_wall": round(main_run["d2h"] / main_run["seconds"] / 1e9, 2),
                 # what bounds `value` in spill mode: both directions of the host link together took 87.7 GB/s on this
                 # hardware (1 GB copies, SDMA in next to the copy kernel out; each direction alone 57.6 / 54.7 GB/s)
                 "both_directions_GBps_over_wall": round((main_run["h2d"] + main_run["d2h"]) / main_run["seconds"] / 1e9, 2),
                 "both_directions_GBps_measured_cap": LINK_CAP_GBPS,
                 "frac_of_link_cap": round((main_run["h2d"] + main_run["d2h"]) / main_run["seconds"] / 1e9 / LINK_CAP_GBPS, 3)},
        "final_losses": [round(x, 4) for x in main_run["losses"]],
    }
    if main_run["overlap"]:
        out["overlap"] = overlap_report(main_run, args.steps)
    if not args.no_extra:
        other = "resident" if args.mode == "spill" else "spill"
        o = measure(cfg, n_models, other, args.steps, args.warmup, False, R, H, torch, pilot=True)
        n_sh = cfg["L"] // cfg["k"] + 2
        out["pilot_costs_us"] = {"forward": [round(x / 1e3, 1) for x in o["pilot_ns"][:n_sh]],
                                 "backward_with_adam": [round(x / 1e3, 1) for x in o["pilot_ns"][n_sh:]],
                                 "shards": "EMBED, block shards 1..S, HEAD; model 0, each task alone on the device"}
        fp = [H.hydra_shard_footprint(H.model_desc(cfg, 1e-4), n) for n in range(0, cfg["L"] + 1)]
        out["partitioner"] = {"footprint_MB_by_layers_in_shard": [round(x / 1e6, 1) for x in fp[1:]],
                              "embed_head_MB": round(fp[0] / 1e6, 1),
                              "cuts_at_bound_of_2_layer_shard": H.hydra_partition(H.model_desc(cfg, 1e-4), max(fp[2], fp[0]))[0]}
        out[other] = {"value": round(tokens_per_step * args.steps / o["seconds"], 1), "unit": "tokens/s",
                      "ms_per_step": round(1e3 * o["seconds"] / args.steps, 3),
                      "host_enqueue_ms_per_step": round(1e3 * o["enqueue_seconds"] / args.steps, 3),
                      "shard_buffers": o["n_slots"]}
        if args.extra_micro > 1 and args.micro == 1:
            # same models, shards and buffers, but every shard visit runs several micro-batches while the shard is
            # resident: the state traffic per step is unchanged and serves that many times the tokens
            steps_m = max(2, args.steps // 2)
            for nm in (args.extra_micro, 2 * args.extra_micro):
                mc = dict(cfg, n_micro=nm)
                o = measure(mc, n_models, "spill", steps_m, 1, False, R, H, torch)
                out[f"spill_micro{nm}"] = {
                    "value": round(tokens_per_step * nm * steps_m / o["seconds"], 1), "unit": "tokens/s",
                    "ms_per_step": round(1e3 * o["seconds"] / steps_m, 3), "tokens_per_step": tokens_per_step * nm,
                    "h2d_GB_per_step": round(o["h2d"] / steps_m / 1e9, 3), "shard_buffers": o["n_slots"],
                    "overlap": overlap_report(o, steps_m)}
            # the same 4x tokens per shard visit as ONE micro-batch of 4x the samples: activation memory grows
            # fourfold (no issue on a 288 GB part), the GEMMs become four times larger and fill the chip
            bc = dict(cfg, B=cfg["B"] * args.extra_micro)
            o = measure(bc, n_models, "spill", steps_m, 1, False, R, H, torch)
            out[f"spill_batch_x{args.extra_micro}"] = {
                "value": round(tokens_per_step * args.extra_micro * steps_m / o["seconds"], 1), "unit": "tokens/s",
                "ms_per_step": round(1e3 * o["seconds"] / steps_m, 3), "tokens_per_step": tokens_per_step * args.extra_micro,
                "batch": bc["B"], "shard_buffers": o["n_slots"], "overlap": overlap_report(o, steps_m)}
        # per-kernel HIP-event timing over the same steps (resident buffers so that copies do not perturb kernels)
        t = measure(cfg, n_models, "resident", args.steps, args.warmup, True, R, H, torch)
        ks = sorted(t["kernels"], key=lambda k: -k["ms"])
        total_ms = sum(k["ms"] for k in ks)
        dom = ks[0]
        if dom["flops"] > 0:
            ach = dom["flops"] / (dom["ms"] * 1e-3) / 1e12
            out["roofline"] = {"bound": "mfma", "achieved": round(ach, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                               "unit": "TFLOP/s", "frac": round(ach / MFMA_BF16_PEAK_TFLOPS, 4),
                               "traffic": measured_traffic(args.config, dom["name"]),
                               "kernel": dom["name"], "launches": dom["launches"],
                               "avg_us": round(1e3 * dom["ms"] / dom["launches"], 2)}
        else:
            ach = dom["bytes"] / (dom["ms"] * 1e-3) / 1e9
            out["roofline"] = {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                               "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": measured_traffic(args.config, dom["name"]),
                               "kernel": dom["name"],
                               "launches": dom["launches"], "avg_us": round(1e3 * dom["ms"] / dom["launches"], 2)}
        out["kernels"] = [
            {"name": k["name"], "launches": k["launches"], "ms_per_step": round(k["ms"] / args.steps, 4),
             "share": round(k["ms"] / total_ms, 4),
             **({"TFLOPs": round(k["flops"] / (k["ms"] * 1e-3) / 1e12, 1)} if k["flops"] > 0 else
                {"GBps": round(k["bytes"] / (k["ms"] * 1e-3) / 1e9, 1)})}
            for k in ks]
        gemm = [k for k in ks if k["flops"] > 0]
        out["gemm_aggregate"] = {"TFLOPs": round(sum(k["flops"] for k in gemm) / (sum(k["ms"] for k in gemm) * 1e-3) / 1e12, 1),
                                 "frac_of_mfma_peak": round(sum(k["flops"] for k in gemm) / (sum(k["ms"] for k in gemm) * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                                 "kernel_ms_per_step": round(total_ms / args.steps, 3)}
        out["block_gemm_large_shapes"] = block_gemm_large_shapes(H, torch)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
