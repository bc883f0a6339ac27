"""Model state in ordinary (pageable) host memory: promotes and write-backs travel through the page-locked staging
ring (hydra_init_desc.stage) on the library's own threads.  The staging tier moves bytes and nothing else, so every
result must equal the page-locked path bit for bit - with rings of 1 MiB chunks, so that a shard takes many chunks
and the ring wraps several times per copy."""
import numpy as np
import pytest

import synth_inputs as SI
from tests.test_gpu_parity import (assert_same_state, check_against_models_alone, costs_of, oracle_order, run_manual,
                                   scheduled_run)

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

STAGE = dict(stage_bytes=16 << 20)        # two rings of eight 1 MiB chunks


@pytest.fixture(scope="module")
def rt():
    from paper_2110_08633_amd import hydra, runtime
    return hydra, runtime


def _cfg(dtype, **kw):
    # embedding / head shards of 5 MB per state array, block shards of 3 MB: several ring chunks each
    c = SI.small_cfg(L=4, d=128, H=2, F=512, V=10007, T=64, B=2, k=2, dtype=dtype, lrs=[1e-4])
    c.update(kw)
    return c


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_pageable_state_step_by_step_against_the_oracle(rt, dtype):
    """Every shard promoted from and written back to ordinary memory, two steps, everything against the oracle, and
    the final state equal to the page-locked path's bit for bit."""
    H, R = rt
    cfg = _cfg(dtype)
    _, staged, loss_s, _ = run_manual(rt, cfg, 2, max_slots=2, flags=H.FLAG_POISON, session_kw=STAGE, pageable=True,
                                      test_id=f"pageable {dtype}")
    _, pinned, loss_p, _ = run_manual(rt, cfg, 2, max_slots=2, flags=H.FLAG_POISON, oracle=False)
    assert_same_state(staged, pinned, "pageable vs page-locked: ")
    assert loss_s == loss_p


@pytest.mark.parametrize("max_slots,lanes,threads", [(2, 1, 1), (3, 2, 3), (0, 2, 2)])
def test_scheduled_run_with_pageable_and_page_locked_models(rt, max_slots, lanes, threads):
    """Three models through the scheduler, the first and the last in ordinary memory and the middle one
    page-locked, with deep prefetch, write-backs right after Adam and buffers reused across models: exact task
    order, and every model equals its run alone (page-locked, compared with the oracle step by step)."""
    H, R = rt
    cfg = _cfg("bf16", n_models=3, lrs=[1e-4, 3e-4, 1e-5])
    n, nmb = 3, [2, 2, 1]
    Ws = [SI.make_weights(cfg, 10 + m) for m in range(n)]
    batches = [[SI.make_batch(cfg, 100 + 10 * m + i) for i in range(nmb[m])] for m in range(n)]
    tables = [costs_of(cfg)] * n
    want, _, _ = oracle_order([cfg] * n, nmb, tables)
    trace, states, losses, st = scheduled_run(rt, [cfg] * n, Ws, cfg["lrs"], batches, nmb, tables, max_slots=max_slots,
                                              lanes=lanes, flags=H.FLAG_POISON,
                                              session_kw=dict(STAGE, stage_threads=threads), pageable=[True, False, True])
    assert trace == want
    if max_slots:
        assert st["bytes_d2h"] == sum(nmb) * 12 * SI.n_params(cfg)
    check_against_models_alone(rt, [cfg] * n, [cfg] * n, Ws, cfg["lrs"], batches, states, losses, "bf16")


def test_tied_head_and_micro_batches_with_pageable_state(rt):
    """The tied LM head takes its copy of wte from the host arrays or from the embedding shard's buffer; with the
    state in ordinary memory the first goes through the staging ring."""
    H, R = rt
    base = _cfg("bf16", tie=True, L=2, k=1)
    cfg = dict(base, n_micro=2)
    big = dict(base, B=base["B"] * 2)
    W = SI.make_weights(base, 31)
    batches = [SI.make_batch(big, 400 + i) for i in range(3)]
    _, pinned, loss_p, _ = run_manual(rt, cfg, 3, max_slots=2, W=W, lr=1e-4, batches=batches, oracle_cfg=big,
                                      test_id="tied, page-locked")
    trace, states, losses, st = scheduled_run(rt, [cfg], [W], [1e-4], [batches], [3], [costs_of(base)], max_slots=3,
                                              session_kw=STAGE, pageable=[True], slots_for_arena=3)
    assert_same_state(states[0], pinned, "tied, pageable, scheduled: ")
    assert losses[0] == loss_p


def test_pageable_state_needs_a_staging_area(rt):
    H, R = rt
    cfg = _cfg("bf16")
    sess = R.Session(R.arena_bytes_for([cfg], 2), max_slots=2)
    with pytest.raises(H.HydraError) as e:
        sess.add_model(cfg, None, 1e-4, pageable=True)
    assert e.value.code == H.E_INVAL
    sess.close()
    with pytest.raises(H.HydraError) as e:      # an area too small for two rings
        R.Session(R.arena_bytes_for([cfg], 2), max_slots=2, stage_bytes=1 << 20)
    assert e.value.code == H.E_INVAL


def test_write_back_mechanisms_agree(rt):
    """Write-backs travel through hipMemcpyAsync or through the library's copy kernel: by default the first for
    page-locked state and the second behind the staging area; either can be forced for both.  They move bytes:
    every combination must leave the same state."""
    H, R = rt
    cfg = _cfg("bf16")
    _, want, loss_w, _ = run_manual(rt, cfg, 2, max_slots=2, flags=H.FLAG_POISON, oracle=False)
    for flag in (H.FLAG_D2H_KERNEL, H.FLAG_D2H_MEMCPY):
        for pageable in (False, True):
            kw = dict(session_kw=STAGE, pageable=True) if pageable else {}
            _, got, loss, _ = run_manual(rt, cfg, 2, max_slots=2, flags=H.FLAG_POISON | flag | (H.FLAG_CKPT_SPILL if pageable else 0),
                                         oracle=False, **kw)
            assert_same_state(got, want, f"write-back flag {flag}, pageable={pageable}: ")
            assert loss == loss_w
    with pytest.raises(H.HydraError) as e:
        R.Session(R.arena_bytes_for([cfg], 2), max_slots=2, flags=H.FLAG_D2H_KERNEL | H.FLAG_D2H_MEMCPY)
    assert e.value.code == H.E_INVAL


@pytest.mark.parametrize("locked", [(True, False, True, False), (False, True, True, True), (True, True, False, None)])
def test_some_arrays_page_locked_and_some_not(rt, locked):
    """What the driver lets a process page-lock may cover some of a model's arrays only: master, m, v and the bf16
    copy are each taken as they come (locked[i]: page-locked or ordinary memory; None: no bf16 copy)."""
    H, R = rt
    cfg = _cfg("bf16")
    W = SI.make_weights(cfg, SI.model_seed(cfg, 0))
    batches = [SI.make_batch(cfg, SI.batch_seed(cfg, 0, i)) for i in range(2)]
    _, want, loss_w, _ = run_manual(rt, cfg, 2, max_slots=2, flags=H.FLAG_POISON, oracle=False)
    sess = R.Session(R.arena_bytes_for([cfg], 2), max_slots=2, flags=H.FLAG_POISON, **STAGE)
    n = H.hydra_model_layout(H.model_desc(cfg, 1e-4)).n_params
    arrays = [sess._host(n, np.uint16 if i == 3 else np.float32, pageable=not locked[i]) if locked[i] is not None else False
              for i in range(4)]
    rec = sess.add_model(cfg, W, cfg["lrs"][0], host=tuple(arrays[:3]), work_copy=arrays[3])
    for tok, tgt in batches:
        loss = sess.train_step_manual(rec, tok, tgt, collect=False)["loss"]
    H.hydra_sync(sess.ctx)
    from tests.test_gpu_parity import host_state
    got = host_state(sess, rec)
    if locked[3] is not None:
        u = rec["master"].view(np.uint32).astype(np.uint64)
        lo = H.hydra_shard_range(rec["desc"], 1)[0]
        hi = sum(H.hydra_shard_range(rec["desc"], rec["S"]))
        assert np.array_equal(rec["work"][lo:hi], ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)[lo:hi])
    sess.close()
    assert_same_state(got, want, f"arrays page-locked {locked}: ")
    assert loss == loss_w
