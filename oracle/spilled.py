"""CPU oracle for the paper's execution method: spilled, shard-by-shard
training of several models interleaved by the Sharded-LRTF scheduler.

TEST INFRASTRUCTURE ONLY; never imported by the product path.

Spilled execution (Section 2.3 of the paper): a model is cut into shards, each
shard is visited twice per minibatch - once forward, once backward.  After a
forward visit only the shard's output activation (the checkpoint at the shard
boundary) is kept; the backward visit recomputes the shard's forward from the
checkpoint at its input, back-propagates the incoming boundary gradient, and
hands the gradient at its input to the next backward visit.  Reading taken
where the paper is silent: Adam runs on a shard's parameters right after that
shard's backward visit (Adam is elementwise and no shard's gradient depends on
another shard's parameters being old or new once its own backward is done, so
this equals stepping after the whole backward pass).

Shard numbering: 0 = embeddings, 1..S = runs of k consecutive blocks,
S+1 = final LayerNorm + LM head + loss.

Sharded-LRTF (Section 2.4): whenever the device is free, take the next shard
task of the model with the longest remaining total time; a shard task is
atomic.  Readings: the remaining time of a model is the summed cost of its
tasks not yet started; ties go to the lowest model index; costs are inputs.
"""
from __future__ import annotations

import numpy as np

from . import decoder as D

FWD, BWD = 0, 1


def shard_tensor_names(cfg, s):
    """Names of the parameter tensors owned by shard s."""
    L, k = cfg["L"], cfg["k"]
    S = L // k
    if s == 0:
        return ["wte", "wpe"]
    if s == S + 1:
        return ["lnf_g", "lnf_b"] if cfg.get("tie") else ["lnf_g", "lnf_b", "w_lm"]
    return [f"h{l}.{n}" for l in range((s - 1) * k, s * k) for n in D.BLOCK_TENSORS]


def model_task_chain(cfg, n_minibatches):
    """[(shard, phase)] for one model: forward visits in shard order, backward
    visits in reverse, repeated per minibatch."""
    S = cfg["L"] // cfg["k"]
    one = [(s, FWD) for s in range(S + 2)] + [(s, BWD) for s in range(S + 1, -1, -1)]
    return one * n_minibatches


def sharded_lrtf(chains, costs):
    """chains[m] = list of tasks of model m in dependency order; costs[m][i] =
    integer cost of chains[m][i].  Returns the executed order as a list of
    (model, index_in_chain)."""
    n = len(chains)
    cursor = [0] * n
    remaining = [int(sum(c)) for c in costs]
    order = []
    while True:
        best = -1
        for m in range(n):
            if cursor[m] < len(chains[m]) and (best < 0 or remaining[m] > remaining[best]):
                best = m
        if best < 0:
            return order
        order.append((best, cursor[best]))
        remaining[best] -= int(costs[best][cursor[best]])
        cursor[best] += 1


class SpilledModel:
    """State of one model under spilled execution.  Parameters and Adam state
    live in 'host' dicts; a visit touches only its own shard's tensors."""

    def __init__(self, cfg, P, lr, dtype):
        self.cfg = cfg
        self.lr = lr
        self.P = D.cast_params(P, dtype)
        self.Mo = D.zeros_like_params(self.P)
        self.Vo = D.zeros_like_params(self.P)
        self.S = cfg["L"] // cfg["k"]
        self.t = 0                      # completed optimizer steps
        self.ckpt = {}                  # boundary index -> activation; boundary b = output of shard b
        self.dbound = None              # gradient flowing into the next backward visit
        self.dlogits = None
        self.dwte_head = None
        self.loss = None
        self.logits = None
        self.grads = {}                 # last gradients, kept only for inspection by tests
        self.tokens = self.targets = None

    def set_batch(self, tokens, targets):
        self.tokens, self.targets = tokens, targets

    # -- forward visit -------------------------------------------------------
    def forward(self, s):
        cfg, P = self.cfg, self.P
        B, T = self.tokens.shape
        if s == 0:
            self.ckpt = {0: D.embed_fwd(self.tokens, P["wte"], P["wpe"])}
        elif s <= self.S:
            x = self.ckpt[s - 1]
            for l in range((s - 1) * cfg["k"], s * cfg["k"]):
                x, _ = D.block_fwd(P, l, x, B, T, cfg["H"])     # intermediates discarded
            self.ckpt[s] = x
        else:
            self.logits, _ = D.head_fwd(P, self.ckpt[self.S])
            self.loss, _ = D.cross_entropy(self.logits, self.targets)

    # -- backward visit (recompute, backprop, Adam on this shard) -------------
    def backward(self, s):
        cfg, P = self.cfg, self.P
        B, T = self.tokens.shape
        G = {}
        if s == self.S + 1:
            logits, hc = D.head_fwd(P, self.ckpt[self.S])
            _, dlogits = D.cross_entropy(logits, self.targets)
            self.dbound, G = D.head_bwd(P, dlogits, hc)
            # tied head: its part of the wte gradient waits for the embedding shard's backward visit
            self.dwte_head = G.pop("wte_head", None)
        elif s >= 1:
            x = self.ckpt[s - 1]
            caches = []
            layers = list(range((s - 1) * cfg["k"], s * cfg["k"]))
            for l in layers:
                x, c = D.block_fwd(P, l, x, B, T, cfg["H"])
                caches.append(c)
            dx = self.dbound
            for l, c in zip(reversed(layers), reversed(caches)):
                dx, g = D.block_bwd(P, l, dx, c, B, T, cfg["H"])
                G.update(g)
            self.dbound = dx
        else:
            G["wte"], G["wpe"] = D.embed_bwd(self.dbound, self.tokens, cfg["V"])
            if self.dwte_head is not None:
                G["wte"] = self.dwte_head + G["wte"]
            self.dbound = None
        if s == self.S + 1:
            self.t += 1                 # first backward visit of a minibatch opens step t
        for name in shard_tensor_names(cfg, s):
            P[name], self.Mo[name], self.Vo[name] = D.adam_update(
                P[name], self.Mo[name], self.Vo[name], G[name], self.t, self.lr)
        self.grads.update(G)

    def run_task(self, s, phase):
        (self.forward if phase == FWD else self.backward)(s)


def run_interleaved(models, batches, order, chains):
    """Execute 'order' (from sharded_lrtf) over SpilledModel objects.
    batches[m][i] = (tokens, targets) of minibatch i of model m."""
    per_mb = [2 * (mm.S + 2) for mm in models]
    for m, idx in order:
        mm = models[m]
        if idx % per_mb[m] == 0:
            mm.set_batch(*batches[m][idx // per_mb[m]])
        s, phase = chains[m][idx]
        mm.run_task(s, phase)
