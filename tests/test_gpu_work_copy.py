"""A bf16 rounding of the master kept on the host (hydra_host_state.work_bf16).  Promotes for forward visits of block
shards then carry that copy and the shard's fp32 vectors instead of the whole fp32 master.  The copy holds exactly
the values the device would derive from the master, so every result must equal the plain path bit for bit; the copy
itself must be the rounding of the final master; the link counters follow closed forms."""
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


def _cfg(**kw):
    c = SI.small_cfg(L=4, d=128, H=2, F=512, V=10007, T=64, B=2, k=2, dtype="bf16", lrs=[1e-4])
    c.update(kw)
    return c


def round_bf16(x):
    """fp32 -> bf16 bits, round to nearest even (plain integer arithmetic on the bit patterns)."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def block_range(rt, cfg):
    H, _ = rt
    desc = H.model_desc(cfg, 1e-4)
    S = cfg["L"] // cfg["k"]
    lo = H.hydra_shard_range(desc, 1)[0]
    off, cnt = H.hydra_shard_range(desc, S)
    return lo, off + cnt


def flatten(rt, cfg, named):
    """Named tensors -> the flat canonical array."""
    H, _ = rt
    desc = H.model_desc(cfg, 1e-4)
    lay = H.hydra_model_layout(desc)
    out = np.zeros(lay.n_params, np.float32)
    for i in range(lay.n_tensors):
        name, off, rows, cols, _ = H.hydra_model_tensor(desc, i)
        out[off:off + rows * cols] = np.asarray(named[name], np.float32).reshape(-1)
    return out


def link_bytes_manual(rt, cfg, steps, work_copy):
    """What train_step_manual moves per run: every shard promoted for its forward visit and evicted (the HEAD shard
    stays for its backward visit), every shard promoted with its Adam state for the backward visit."""
    H, _ = rt
    desc = H.model_desc(cfg, 1e-4)
    S = cfg["L"] // cfg["k"]
    c = [H.hydra_shard_range(desc, s)[1] for s in range(S + 2)]
    vec = cfg["k"] * (9 * cfg["d"] + cfg["F"])                 # fp32 vectors of a block shard
    fwd = [4 * x for x in c]
    if work_copy:
        for s in range(1, S + 1):
            fwd[s] = 2 * c[s] + 4 * vec
    h2d = sum(fwd) + 12 * sum(c[:-1]) + 8 * c[-1]
    d2h = 12 * sum(c)                                          # the copy never crosses the link on its way back
    return steps * h2d, steps * d2h


@pytest.mark.parametrize("pageable", [False, True])
def test_forward_promotes_from_the_bf16_copy_change_nothing(rt, pageable):
    H, R = rt
    cfg = _cfg()
    kw = dict(session_kw=STAGE, pageable=True) if pageable else {}
    ex = {}
    _, with_copy, loss_c, _ = run_manual(rt, cfg, 3, max_slots=2, flags=H.FLAG_POISON, work_copy=True, extras=ex,
                                         test_id=f"bf16 host copy, {'ordinary' if pageable else 'page-locked'} memory", **kw)
    plain_ex = {}
    _, plain, loss_p, _ = run_manual(rt, cfg, 3, max_slots=2, flags=H.FLAG_POISON, oracle=False, extras=plain_ex)
    assert_same_state(with_copy, plain, "with the bf16 host copy vs without: ")
    assert loss_c == loss_p
    # the copy: block shards follow the master, the other shards keep the rounding made at registration
    lo, hi = block_range(rt, cfg)
    w = flatten(rt, cfg, with_copy[0])
    assert np.array_equal(ex["work"][lo:hi], round_bf16(w[lo:hi]))
    w0 = flatten(rt, cfg, SI.make_weights(cfg, SI.model_seed(cfg, 0)))
    assert np.array_equal(ex["work"][:lo], round_bf16(w0[:lo])) and np.array_equal(ex["work"][hi:], round_bf16(w0[hi:]))
    assert not np.array_equal(ex["work"][lo:hi], round_bf16(w0[lo:hi]))
    # link traffic; run_manual reads gradients back, which the counters do not include
    h2d, d2h = link_bytes_manual(rt, cfg, 3, True)
    assert (ex["stats"]["bytes_h2d"], ex["stats"]["bytes_d2h"]) == (h2d, d2h)
    h2d0, d2h0 = link_bytes_manual(rt, cfg, 3, False)
    assert (plain_ex["stats"]["bytes_h2d"], plain_ex["stats"]["bytes_d2h"]) == (h2d0, d2h0)
    assert h2d < h2d0


@pytest.mark.parametrize("max_slots,lanes,threads", [(2, 1, 1), (3, 2, 3), (0, 2, 2)])
def test_scheduled_models_with_and_without_the_bf16_copy(rt, max_slots, lanes, threads):
    """Three models through the scheduler: ordinary memory with the copy, page-locked with the copy, page-locked
    without; buffers reused across models, and (max_slots 0) shards that stay resident between their forward and
    their backward visit, which then fetches the master into a buffer that holds only the bf16 copy.  Exact task
    order, and every model equals its run alone without the copy (compared with the oracle step by step)."""
    H, R = rt
    cfg = _cfg(n_models=3, lrs=[1e-4, 3e-4, 1e-5])
    n, nmb = 3, [2, 2, 1]
    Ws = [SI.make_weights(cfg, 20 + m) for m in range(n)]
    batches = [[SI.make_batch(cfg, 200 + 10 * m + i) for i in range(nmb[m])] for m in range(n)]
    tables = [costs_of(cfg)] * n
    want, _, _ = oracle_order([cfg] * n, nmb, tables)
    ex = {}
    trace, states, losses, st = scheduled_run(rt, [cfg] * n, Ws, cfg["lrs"], batches, nmb, tables, max_slots=max_slots,
                                              lanes=lanes, flags=H.FLAG_POISON,
                                              session_kw=dict(STAGE, stage_threads=threads),
                                              pageable=[True, False, False], work_copy=[True, True, False], extras=ex)
    assert trace == want
    lo, hi = block_range(rt, cfg)
    for m in range(2):
        assert np.array_equal(ex["work"][m][lo:hi], round_bf16(flatten(rt, cfg, states[m][0])[lo:hi])), \
            f"model {m}: stale bf16 copy"
    assert ex["work"][2] is None
    if max_slots:
        assert st["bytes_d2h"] == sum(nmb) * 12 * SI.n_params(cfg)      # every minibatch writes every shard back once
    check_against_models_alone(rt, [cfg] * n, [cfg] * n, Ws, cfg["lrs"], batches, states, losses, "bf16")


def test_micro_batches_and_checkpoint_spill_with_the_bf16_copy(rt):
    """Several micro-batches per visit and boundary activations through host memory, one-layer shards."""
    H, R = rt
    base = _cfg(L=3, k=1)
    cfg = dict(base, n_micro=2)
    big = dict(base, B=base["B"] * 2)
    W = SI.make_weights(base, 41)
    batches = [SI.make_batch(big, 500 + i) for i in range(2)]
    flags = H.FLAG_POISON | H.FLAG_CKPT_SPILL
    _, plain, loss_p, _ = run_manual(rt, cfg, 2, max_slots=2, W=W, lr=1e-4, batches=batches, oracle_cfg=big, flags=flags,
                                     test_id="micro-batches, checkpoints spilled, no copy")
    for pageable in (False, True):
        kw = dict(session_kw=STAGE, pageable=True) if pageable else {}
        _, got, loss, _ = run_manual(rt, cfg, 2, max_slots=2, W=W, lr=1e-4, batches=batches, oracle_cfg=big, flags=flags,
                                     oracle=False, work_copy=True, **kw)
        assert_same_state(got, plain, f"bf16 copy, pageable={pageable}: ")
        assert loss == loss_p


def test_fp32_models_ignore_the_copy_and_page_locked_state_needs_a_page_locked_copy(rt):
    H, R = rt
    cfg = _cfg(dtype="f32")
    ex = {}
    run_manual(rt, cfg, 1, max_slots=2, oracle=False, work_copy=True, extras=ex)
    assert (ex["stats"]["bytes_h2d"], ex["stats"]["bytes_d2h"]) == link_bytes_manual(rt, cfg, 1, False)
    cfg = _cfg()
    sess = R.Session(R.arena_bytes_for([cfg], 2), max_slots=2)
    desc = H.model_desc(cfg, 1e-4)
    n = H.hydra_model_layout(desc).n_params
    master, m, v = (sess._host(n) for _ in range(3))
    stage = sess._host(4 * cfg["B"] * cfg["T"], np.int32)
    with pytest.raises(H.HydraError) as e:
        H.hydra_register_model(sess.ctx, desc, master, m, v, None, stage, np.zeros(n, np.uint16))
    assert e.value.code == H.E_INVAL
    sess.close()


def test_runtime_streams_and_caller_arena(rt):
    """The runtime's stream set is chosen once per count, holds distinct streams, and two of its first four do not
    hold each other up; a context can run in a caller's device buffer, and one that is too small is refused."""
    H, R = rt
    four = R.independent_streams(4)
    assert len(four) == 4 and len({s.cuda_stream for s in four}) == 4
    assert R.independent_streams(4) is four
    x = torch.zeros(64, device="cuda")
    for a, b in ((four[0], four[1]), (four[2], four[3]), (four[0], four[3])):
        torch.cuda.synchronize()
        ea, eb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(a):
            torch.cuda._sleep(2_500_000)
            ea.record(a)
        with torch.cuda.stream(b):
            x.add_(1.0)
            eb.record(b)
        torch.cuda.synchronize()
        assert eb.elapsed_time(ea) > 0.25, "a small kernel on one stream waited for the spin kernel on another"
    cfg = _cfg()
    need = R.arena_bytes_for([cfg], 2)
    buf = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(ValueError):
        R.Session(need, max_slots=2, arena=buf[: need // 2])
    results = []
    for arena in (buf, None):
        sess = R.Session(need, max_slots=2, arena=arena)
        rec = sess.add_model(cfg, SI.make_weights(cfg, 5), 1e-4)
        tok, tgt = SI.make_batch(cfg, 6)
        results.append(sess.train_step_manual(rec, tok, tgt, collect=False)["loss"])
        sess.close()
    assert results[0] == results[1]
