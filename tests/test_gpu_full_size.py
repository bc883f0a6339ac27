"""Parity at the full sizes of the reference workloads, in the launch configuration bench.py times (bf16 MFMA
path, shard buffers cycled through promote / demote): one whole training step of a GPT-2-small-shaped model,
and depth-reduced copies (one block shard, full widths, vocabulary and sequence length) of the larger
workloads.  The oracle (float64) computes every output, so everything is compared, not a sample."""
import numpy as np
import pytest

import synth_inputs as SI
from tests.test_gpu_parity import TOL, check_step, check_weights, oracle_steps, update_ill

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def run_one_step(cfg, max_slots=3):
    from paper_2110_08633_amd import hydra as H, runtime as R
    W = SI.make_weights(cfg, SI.model_seed(cfg, 0))
    lr = cfg["lrs"][0]
    batches = [SI.make_batch(cfg, SI.batch_seed(cfg, 0, 0))]
    refs, _, _, _ = oracle_steps(cfg, W, lr, batches)
    sess = R.Session(R.arena_bytes_for([cfg], max_slots), max_slots=max_slots)
    rec = sess.add_model(cfg, W, lr)
    got = sess.train_step_manual(rec, *batches[0])
    H.hydra_sync(sess.ctx)
    after = sess.unpack(rec, rec["master"])
    check_step(cfg, got, refs[0], TOL[cfg["dtype"]])
    ill = update_ill({}, refs[0]["grads"], cfg["dtype"])
    check_weights(after, refs[0]["after"], refs[0]["before"], ill, lr, 1, cfg["dtype"])
    assert abs(refs[0]["loss"] - np.log(cfg["V"])) < 1.0        # random init: close to ln V
    sess.close()


def test_gpt2_small_full_size_one_step():
    """12 layers, d 768, 12 heads, MLP 3072, vocab 50257, seq 512, batch 4, 2-layer shards."""
    run_one_step(SI.CONFIGS["gpt2s"])


@pytest.mark.parametrize("name", ["gpt2m", "gpt2xl", "gpt6b"])
def test_large_widths_depth_reduced(name):
    """Same d, heads, MLP width, vocabulary, sequence and batch as the workload; depth cut to one block shard."""
    cfg = dict(SI.CONFIGS[name])
    cfg["L"] = cfg["k"]
    run_one_step(cfg, max_slots=2)
