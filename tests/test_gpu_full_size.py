"""Parity at the full sizes of the reference workloads, in the launch configuration bench.py times (bf16 MFMA
path, shard buffers cycled through promote / demote, every shard spilled to pinned host memory between visits):
  * GPT-2 small (BASELINE config 2) and GPT-2 medium (config 3) at full depth, one model, one step, every output
    compared with the float64 oracle;
  * four GPT-2-medium-width models with two 4-layer shards each through the scheduler (exact task order);
  * GPT-2 XL widths (config 4), four models with two 6-layer shards each under the 24 GB shard-buffer cap;
  * the 6 B-parameter widths (config 5), two models with two 2-layer shards each on two shard buffers, with one and
    with two compute lanes.
Depth is cut (to two block shards, so that a block-shard -> block-shard boundary exists) only where the oracle
would otherwise take many minutes; widths, heads, vocabulary, sequence length and batch are the workload's."""
import numpy as np
import pytest

import synth_inputs as SI
from tests.test_gpu_parity import (check_against_models_alone, costs_of, oracle_order, run_manual, scheduled_run)

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def rt():
    from paper_2110_08633_amd import hydra, runtime
    return hydra, runtime


def test_gpt2_small_full_size_one_step(rt):
    """12 layers, d 768, 12 heads, MLP 3072, vocab 50257, seq 512, batch 4, 2-layer shards, three shard buffers."""
    cfg = SI.CONFIGS["gpt2s"]
    refs, _, _, _ = run_manual(rt, cfg, 1, max_slots=3, test_id="gpt2s full size")
    assert abs(refs[0]["loss"] - np.log(cfg["V"])) < 1.0        # random init: close to ln V


def test_gpt2_medium_full_depth_one_step(rt):
    """BASELINE config 3 as stated, one of its models: 24 layers, d 1024, 16 heads, MLP 4096, vocab 50257, seq
    1024, batch 2, six 4-layer shards spilled to pinned host memory between uses, three shard buffers."""
    cfg = SI.CONFIGS["gpt2m"]
    refs, _, _, _ = run_manual(rt, cfg, 1, max_slots=3, test_id="gpt2m full depth")
    assert abs(refs[0]["loss"] - np.log(cfg["V"])) < 1.0


def _models(name, n_models, L):
    cfg = dict(SI.CONFIGS[name], L=L, n_models=n_models)
    cfg["lrs"] = cfg["lrs"][:n_models]
    Ws = [SI.make_weights(cfg, SI.model_seed(cfg, m)) for m in range(n_models)]
    batches = [[SI.make_batch(cfg, SI.batch_seed(cfg, m, 0))] for m in range(n_models)]
    return cfg, Ws, batches


def test_four_gpt2_medium_models_scheduled(rt):
    """Config 3's four models (different learning rates and weights) with two 4-layer shards each, alternated by
    Sharded-LRTF on two lanes with six shard buffers: exact task order, and every model equals its run alone, which
    equals the oracle."""
    H, R = rt
    n = 4
    cfg, Ws, batches = _models("gpt2m", n, 8)
    tables = [costs_of(cfg)] * n
    want, _, _ = oracle_order([cfg] * n, [1] * n, tables)
    trace, states, losses, st = scheduled_run(rt, [cfg] * n, Ws, cfg["lrs"], batches, [1] * n, tables, max_slots=6,
                                              lanes=2, slots_for_arena=6)
    assert trace == want and st["n_slots"] == 6
    assert st["bytes_d2h"] == n * 12 * SI.n_params(cfg)         # every shard's state went back exactly once
    check_against_models_alone(rt, [cfg] * n, [cfg] * n, Ws, cfg["lrs"], batches, states, losses, "bf16", what="gpt2m x4 ")


def test_gpt2_xl_models_under_the_24_GB_buffer_cap(rt):
    """Config 4's shard-buffer cap: four GPT-2-XL-width models (d 1600, 25 heads, MLP 6400, seq 1024, batch 1) with
    two 6-layer shards each; shard_buffer_cap_bytes = 24 GB decides the number of buffers (6 of 3.7 GB for 16
    shards).  Model 0 is also compared with the oracle."""
    H, R = rt
    n = 4
    cfg, Ws, batches = _models("gpt2xl", n, 12)
    tables = [costs_of(cfg)] * n
    want, _, _ = oracle_order([cfg] * n, [1] * n, tables)
    cap = 24 * 10 ** 9
    trace, states, losses, st = scheduled_run(rt, [cfg] * n, Ws, cfg["lrs"], batches, [1] * n, tables, lanes=2, cap=cap,
                                              slots_for_arena=7)
    assert st["n_slots"] == cap // st["slot_bytes"] == 6
    assert trace == want
    check_against_models_alone(rt, [cfg] * n, [cfg] * n, Ws, cfg["lrs"], batches, states, losses, "bf16",
                               what="gpt2xl x4 ", oracle_models=[0])


_GPT6B_ALONE = {}


def _gpt6b_alone(rt, m, cfg, W, batches, oracle):
    """Model m of the two 6 B-width models run alone through the shard calls on two buffers (kept for the scheduled
    cases below: the run alone does not depend on the lane count)."""
    if m not in _GPT6B_ALONE:
        _GPT6B_ALONE[m] = run_manual(rt, cfg, 1, W=W, lr=cfg["lrs"][m], batches=batches, max_slots=2,
                                     test_id=f"gpt6b model {m}", oracle=oracle)[1:3]
    return _GPT6B_ALONE[m]


def test_gpt6b_model_alone_against_the_oracle(rt):
    """One model of the 6 B-parameter widths (d 4096, 32 heads of 128, MLP 16384, vocab 50400, seq 1024, batch 1)
    with two 2-layer shards on TWO shard buffers of 8 GB, all state in pinned host memory: logits, loss, gradients,
    updated weights, deltas and Adam state against the oracle."""
    cfg, Ws, batches = _models("gpt6b", 1, 4)
    final, loss = _gpt6b_alone(rt, 0, cfg, Ws[0], batches[0], oracle=True)
    assert abs(loss - np.log(cfg["V"])) < 1.0


@pytest.mark.parametrize("lanes", [1, 2])
def test_gpt6b_models_on_two_shard_buffers(rt, lanes):
    """Config 5's buffer cap: two models of the 6 B-parameter widths with two 2-layer shards each, alternated by the
    scheduler on TWO shard buffers, with one and with two compute lanes.  Exact task order; every model equals its
    run alone bit for bit (model 0's run alone is the one compared with the oracle above)."""
    from tests.test_gpu_parity import assert_same_state
    n = 2
    cfg, Ws, batches = _models("gpt6b", n, 4)
    tables = [costs_of(cfg)] * n
    want, _, _ = oracle_order([cfg] * n, [1] * n, tables)
    trace, states, losses, st = scheduled_run(rt, [cfg] * n, Ws, cfg["lrs"], batches, [1] * n, tables, max_slots=2,
                                              lanes=lanes, slots_for_arena=2)
    assert st["n_slots"] == 2 and trace == want
    assert st["bytes_d2h"] == n * 12 * SI.n_params(cfg)
    for m in range(n):
        final, loss = _gpt6b_alone(rt, m, cfg, Ws[m], batches[m], oracle=False)
        assert_same_state(states[m], final, f"gpt6b model {m}: ")
        assert losses[m] == loss
        assert abs(loss - np.log(cfg["V"])) < 1.0
