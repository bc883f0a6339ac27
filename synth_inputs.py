"""Seeded synthetic inputs for GPT-2-shaped multi-model training workloads.

This module is the only code shared between the CPU oracle and the HIP path.
It holds no arithmetic of the method: it only draws random numbers and names
shapes.  Weights come back as a dict of named float32 arrays, batches as int32
token / target arrays; each side packs them into its own storage.

The paper fine-tunes HuggingFace GPT-2 on WikiText-2 (Section 3, "Dataset and
Workload"); neither is available offline, so GPT-2-shaped models with seeded
N(0, 0.02) weights and uniform random token ids stand in for them.
"""
from __future__ import annotations

import numpy as np

# name -> dict(L, d, H, F, V, T, B, k, dtype, n_models, lrs, wseed, dseed)
# dtype: "f32" = fp32 compute, "bf16" = bf16 compute with fp32 master weights.
CONFIGS = {
    # the five workloads of the build contract
    "tiny": dict(L=2, d=128, H=4, F=512, V=512, T=64, B=2, k=1, dtype="f32",
                 n_models=1, lrs=[1e-4], wseed=1000, dseed=501000),
    "gpt2s": dict(L=12, d=768, H=12, F=3072, V=50257, T=512, B=4, k=2, dtype="bf16",
                  n_models=2, lrs=[1e-4, 3e-5], wseed=2000, dseed=502000),
    "gpt2m": dict(L=24, d=1024, H=16, F=4096, V=50257, T=1024, B=2, k=4, dtype="bf16",
                  n_models=4, lrs=[3e-4, 1e-4, 5e-5, 1e-5], wseed=3000, dseed=503000),
    "gpt2xl": dict(L=48, d=1600, H=25, F=6400, V=50257, T=1024, B=1, k=6, dtype="bf16",
                   n_models=4, lrs=[3e-4, 1e-4, 5e-5, 1e-5], wseed=4000, dseed=504000),
    "gpt6b": dict(L=28, d=4096, H=32, F=16384, V=50400, T=1024, B=1, k=2, dtype="bf16",
                  n_models=2, lrs=[1e-4, 3e-5], wseed=5000, dseed=505000),
}

ADAM_BETA1 = 0.9
ADAM_BETA2 = 0.999
ADAM_EPS = 1e-8
INIT_STD = 0.02


def tensor_shapes(cfg):
    """Ordered list of (name, shape, kind) for every parameter tensor.

    kind is "matrix" (weights, embeddings), "bias" or "gain"; the order is the
    canonical one: embeddings, blocks in depth order, final LayerNorm, LM head.
    All matrices are [in, out] so that y = x @ W + b.  With cfg["tie"] the LM
    head has no matrix of its own: logits = z @ wte^T.
    """
    L, d, F, V, T = cfg["L"], cfg["d"], cfg["F"], cfg["V"], cfg["T"]
    out = [("wte", (V, d), "matrix"), ("wpe", (T, d), "matrix")]
    for l in range(L):
        p = f"h{l}."
        out += [
            (p + "ln1_g", (d,), "gain"), (p + "ln1_b", (d,), "bias"),
            (p + "w_qkv", (d, 3 * d), "matrix"), (p + "b_qkv", (3 * d,), "bias"),
            (p + "w_o", (d, d), "matrix"), (p + "b_o", (d,), "bias"),
            (p + "ln2_g", (d,), "gain"), (p + "ln2_b", (d,), "bias"),
            (p + "w_fc", (d, F), "matrix"), (p + "b_fc", (F,), "bias"),
            (p + "w_proj", (F, d), "matrix"), (p + "b_proj", (d,), "bias"),
        ]
    out += [("lnf_g", (d,), "gain"), ("lnf_b", (d,), "bias")]
    if not cfg.get("tie"):
        out += [("w_lm", (d, V), "matrix")]
    return out


def n_params(cfg):
    return int(sum(int(np.prod(s)) for _, s, _ in tensor_shapes(cfg)))


def make_weights(cfg, seed, nontrivial=True):
    """Dict name -> float32 array.  Matrices ~ N(0, 0.02).

    nontrivial=True (parity runs): biases ~ N(0, 0.02) and gains ~ 1 + N(0, 0.02)
    so that every code path sees values that would expose an indexing slip;
    nontrivial=False gives zero biases and unit gains.
    """
    rng = np.random.default_rng(seed)
    w = {}
    for name, shape, kind in tensor_shapes(cfg):
        if kind == "matrix" or nontrivial:
            a = rng.standard_normal(shape, dtype=np.float32) * np.float32(INIT_STD)
            if kind == "gain":
                a += np.float32(1.0)
        else:
            a = np.ones(shape, np.float32) if kind == "gain" else np.zeros(shape, np.float32)
        w[name] = a
    return w


def make_batch(cfg, seed, zipf=False):
    """tokens, targets: int32 [B, T].  targets are the tokens shifted left by
    one; the last position of every sample has target -1 (ignored by the loss).
    zipf=True draws ids from a heavy-tailed distribution (many repeats), which
    stresses the embedding-gradient accumulation."""
    rng = np.random.default_rng(seed)
    B, T, V = cfg["B"], cfg["T"], cfg["V"]
    if zipf:
        tok = np.minimum(rng.zipf(1.3, size=(B, T)) - 1, V - 1).astype(np.int32)
    else:
        tok = rng.integers(0, V, size=(B, T), dtype=np.int32)
    tgt = np.full((B, T), -1, np.int32)
    tgt[:, :-1] = tok[:, 1:]
    return tok, tgt


def model_seed(cfg, m):
    return cfg["wseed"] + m


def batch_seed(cfg, m, step):
    return cfg["dseed"] + 10 * m + step


def n_block_shards(cfg):
    assert cfg["L"] % cfg["k"] == 0
    return cfg["L"] // cfg["k"]


def task_costs(cfg):
    """Integer cost per shard task, in units of 1e6 flops, used as the
    time estimate by the shard-alternating scheduler.  Returned as
    (fwd_cost[S+2], bwd_cost[S+2]) over shards EMBED, blocks 1..S, HEAD.
    The cost table is an input to both sides (the paper takes it from a pilot
    pass, Section 2.2)."""
    L, d, F, V, T, B, k = (cfg[x] for x in ("L", "d", "F", "V", "T", "B", "k"))
    M = B * T
    S = L // k
    blk = 2 * M * d * (3 * d) + 2 * M * d * d + 4 * M * d * F + 2 * B * d * T * (T + 1)
    head = 2 * M * d * V
    emb = M * d
    u = 10 ** 6
    fwd = [max(1, emb // u)] + [max(1, k * blk // u)] * S + [max(1, head // u)]
    bwd = [max(1, emb // u)] + [max(1, 3 * k * blk // u)] * S + [max(1, 2 * head // u)]
    return fwd, bwd


def small_cfg(**kw):
    """A small configuration for tests; defaults give a 2-layer toy model."""
    c = dict(L=2, d=16, H=2, F=64, V=32, T=8, B=2, k=1, dtype="f32",
             n_models=1, lrs=[1e-3], wseed=7, dseed=77)
    c.update(kw)
    return c
