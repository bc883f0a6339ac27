"""Whole-path parity on the GPU: logits, loss, every gradient tensor, every
updated weight tensor and every weight delta of the HIP path against the CPU
oracle (float64 instance) on the same seeded inputs; task order against the
oracle's Sharded-LRTF.  Tolerances: 1e-4 for the fp32 path, 2e-2 for the bf16
path, per tensor as max|a-b|/max|b| and ||a-b||/||b||; integer work exact."""
import numpy as np
import pytest

import synth_inputs as SI
from oracle import decoder as D
from oracle import spilled as SP
from tests.parity_utils import assert_close, rel_errs

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

TOL = {"f32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def rt():
    from paper_2110_08633_amd import hydra, runtime
    return hydra, runtime


def oracle_steps(cfg, W, lr, batches, dtype=np.float64):
    P = D.cast_params(W, dtype)
    Mo, Vo = D.zeros_like_params(P), D.zeros_like_params(P)
    outs = []
    for t, (tok, tgt) in enumerate(batches, 1):
        before = {k: v.copy() for k, v in P.items()}
        o = D.train_step(P, Mo, Vo, tok, tgt, cfg, lr, t)
        o["before"] = before
        o["after"] = {k: v.copy() for k, v in P.items()}
        outs.append(o)
    return outs, P, Mo, Vo


# Adam's first steps move a weight by about lr * g / |g|: where the gradient of an element is at the noise level of
# the arithmetic (e.g. the key bias, whose exact gradient is zero), the step is decided by rounding noise on either
# side.  The gradient check admits an absolute error of tol * max|g| per element, so elements whose oracle gradient is
# below FLOOR = 5 * tol times max|g| of their tensor at any step so far are called ill-conditioned: they may differ by
# a full Adam step; all other elements must meet the tolerance.
FLOOR = {"f32": 5e-4, "bf16": 1e-1}
DELTA_TOL = {"f32": 2e-3, "bf16": 5e-2}


def update_ill(ill, grads, dtype):
    for name, g in grads.items():
        a = np.abs(g)
        bad = a < FLOOR[dtype] * a.max()
        ill[name] = bad if name not in ill else (ill[name] | bad)
    return ill


def check_weights(after_gpu, ref_after, ref_before_first, ill, lr, steps, dtype, what=""):
    tol = TOL[dtype]
    for name, ref in ref_after.items():
        got = after_gpu[name].astype(np.float64)
        assert np.isfinite(got).all(), f"{what}weight {name}: non-finite"
        err = np.abs(got - ref)
        allowed = tol * np.abs(ref).max() + np.where(ill[name], 2.5 * lr * steps, 0.0)
        assert (err <= allowed).all(), f"{what}weight {name}: max excess {(err - allowed).max():.3e}"
        well = ~ill[name]
        if well.any():
            dref = (ref - ref_before_first[name])[well]
            dgot = (got - ref_before_first[name])[well]
            em, e2 = rel_errs(dgot, dref)
            assert e2 <= DELTA_TOL[dtype], f"{what}delta {name}: l2-rel {e2:.3e} (max-rel {em:.3e})"


def check_step(cfg, got, ref, tol):
    assert_close(got["logits"], ref["logits"], tol, "logits")
    assert abs(got["loss"] - ref["loss"]) <= tol * abs(ref["loss"]), ("loss", got["loss"], ref["loss"])
    for name, g in ref["grads"].items():
        assert_close(got["grads"][name], g, tol, f"grad {name}")


def run_manual(rt, cfg, n_steps, flags=0, max_slots=0, zipf=False):
    H, R = rt
    W = SI.make_weights(cfg, SI.model_seed(cfg, 0))
    lr = cfg["lrs"][0]
    batches = [SI.make_batch(cfg, SI.batch_seed(cfg, 0, i), zipf=zipf) for i in range(n_steps)]
    refs, P, Mo, Vo = oracle_steps(cfg, W, lr, batches)
    sess = R.Session(R.arena_bytes_for([cfg], 4, bool(flags & H.FLAG_CKPT_SPILL)), flags=flags, max_slots=max_slots or 4)
    rec = sess.add_model(cfg, W, lr)
    bf16 = cfg["dtype"] == "bf16"
    ill = {}
    for i, (tok, tgt) in enumerate(batches):
        got = sess.train_step_manual(rec, tok, tgt)
        H.hydra_sync(sess.ctx)
        after = {k: v.copy() for k, v in sess.unpack(rec, rec["master"]).items()}
        check_step(cfg, got, refs[i], TOL[cfg["dtype"]])
        update_ill(ill, refs[i]["grads"], cfg["dtype"])
        check_weights(after, refs[i]["after"], refs[0]["before"], ill, lr, i + 1, cfg["dtype"], f"step {i}: ")
    if not bf16:
        for name, a in sess.unpack(rec, rec["m"]).items():
            assert_close(a, Mo[name], 1e-4, f"adam m {name}")
        for name, a in sess.unpack(rec, rec["v"]).items():
            assert_close(a, Vo[name], 2e-4, f"adam v {name}")
    sess.close()
    return refs


def test_tiny_config_fp32_three_steps(rt):
    """BASELINE config 1: 2 layers, d 128, 4 heads, MLP 512, vocab 512, seq 64, batch 2, 1 layer per shard."""
    refs = run_manual(rt, SI.CONFIGS["tiny"], 3)
    assert abs(refs[0]["loss"] - np.log(512)) < 5e-2


@pytest.mark.parametrize("kw", [
    dict(L=2, d=72, H=3, F=136, V=1001, T=72, B=3, k=2),          # ragged everywhere, odd vocabulary
    dict(L=4, d=64, H=8, F=256, V=300, T=264, B=1, k=2),          # T crosses the 256-wide diagonal block
    dict(L=1, d=8, H=1, F=8, V=9, T=8, B=1, k=1),                 # smallest legal shapes
    dict(L=2, d=128, H=2, F=256, V=211, T=200, B=2, k=1),         # head width 64: fused attention on the bf16 path
    dict(L=2, d=128, H=1, F=128, V=97, T=72, B=1, k=2),           # head width 128
])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ragged_shapes(rt, kw, dtype):
    cfg = SI.small_cfg(dtype=dtype, lrs=[1e-4], **kw)       # the learning rate of the reference workloads
    run_manual(rt, cfg, 2)


def test_repeated_tokens_accumulate_exactly(rt):
    """Embedding gradient with many repeated ids (heavy-tailed ids): fp32 path."""
    cfg = SI.small_cfg(L=1, d=64, H=2, F=128, V=50, T=128, B=4, k=1, dtype="f32")
    run_manual(rt, cfg, 1, zipf=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_checkpoint_spill_and_poison_flags(rt, dtype):
    H, _ = rt
    cfg = SI.small_cfg(L=4, d=64, H=2, F=128, V=200, T=64, B=2, k=1, dtype=dtype)
    run_manual(rt, cfg, 2, flags=H.FLAG_CKPT_SPILL | H.FLAG_POISON, max_slots=2)


def test_embedding_forward_is_bit_exact_and_absent_rows_untouched(rt):
    H, R = rt
    cfg = SI.small_cfg(L=1, d=64, H=2, F=128, V=997, T=64, B=2, k=1, dtype="f32")
    W = SI.make_weights(cfg, 5)
    tok, tgt = SI.make_batch(cfg, 6)
    sess = R.Session(R.arena_bytes_for([cfg], 4), max_slots=4)
    rec = sess.add_model(cfg, W, 1e-3)
    sess.train_step_manual(rec, tok, tgt, spill=True)
    H.hydra_sync(sess.ctx)
    x0 = sess.read_act(rec, 0, H.RD_CKPT)
    ref = D.embed_fwd(tok, W["wte"], W["wpe"])                    # float32 instance: one add per element
    assert (x0 == ref).all()
    after = sess.unpack(rec, rec["master"])
    absent = np.setdiff1d(np.arange(cfg["V"]), np.unique(tok))
    assert (after["wte"][absent] == W["wte"][absent]).all()
    assert (sess.unpack(rec, rec["m"])["wte"][absent] == 0).all()
    assert (after["wte"][np.unique(tok)] != W["wte"][np.unique(tok)]).any()
    sess.close()


@pytest.mark.parametrize("max_slots,lanes", [(2, 1), (3, 1), (0, 1), (3, 2), (0, 3)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_scheduled_multi_model_run_matches_oracle(rt, max_slots, lanes, dtype):
    """Three models with different learning rates and weights, interleaved by the library's scheduler with
    prefetch and write-back, against the oracle's interleaved spilled run; task order must be identical."""
    H, R = rt
    cfg = SI.small_cfg(L=4, d=64, H=4, F=256, V=211, T=64, B=2, k=2, dtype=dtype, n_models=3,
                       lrs=[1e-3, 3e-4, 1e-4])
    n, nmb = 3, [2, 1, 2]
    Ws = [SI.make_weights(cfg, 40 + m) for m in range(n)]
    batches = [[SI.make_batch(cfg, 700 + 10 * m + i) for i in range(nmb[m])] for m in range(n)]
    fc, bc = SI.task_costs(cfg)
    chains = [SP.model_task_chain(cfg, nmb[m]) for m in range(n)]
    costs = [[(fc if ph == SP.FWD else bc)[s] for s, ph in ch] for ch in chains]
    order = SP.sharded_lrtf(chains, costs)
    oracle = [SP.SpilledModel(cfg, Ws[m], cfg["lrs"][m], np.float64) for m in range(n)]
    SP.run_interleaved(oracle, batches, order, chains)

    sess = R.Session(R.arena_bytes_for([cfg] * n, 12, lanes=lanes), max_slots=max_slots, lanes=lanes,
                     flags=H.FLAG_POISON if lanes > 1 else 0)
    recs = [sess.add_model(cfg, Ws[m], cfg["lrs"][m]) for m in range(n)]
    sch = H.hydra_sched_create(sess.ctx, [r["id"] for r in recs], nmb, [list(fc) + list(bc)] * n)
    toks = [np.stack([b[0] for b in batches[m]]) for m in range(n)]
    tgts = [np.stack([b[1] for b in batches[m]]) for m in range(n)]
    trace, done = H.hydra_sched_run(sch, toks, tgts, sess.ctx, trace_cap=4096)
    sess.flush()
    S = cfg["L"] // cfg["k"]
    per = 2 * (S + 2)
    assert trace == [(m, chains[m][i][0], chains[m][i][1], i // per) for m, i in order]      # exact
    tol = TOL[dtype]
    for m in range(n):
        assert abs(H.hydra_get_loss(sess.ctx, recs[m]["id"]) - oracle[m].loss) <= tol * oracle[m].loss
        after = sess.unpack(recs[m], recs[m]["master"])
        # gradients of every step from the plain (unsharded) oracle, to mark ill-conditioned elements
        refs, P, _, _ = oracle_steps(cfg, Ws[m], cfg["lrs"][m], batches[m])
        ill = {}
        for r in refs:
            update_ill(ill, r["grads"], dtype)
        for name in P:
            assert (P[name] == oracle[m].P[name]).all()       # interleaved spilled oracle == plain oracle
        check_weights(after, oracle[m].P, refs[0]["before"], ill, cfg["lrs"][m], nmb[m], dtype, f"model {m} ")
    st = H.hydra_get_stats(sess.ctx)
    assert st["n_tasks"] == done == len(order)
    H.hydra_sched_destroy(sch)
    sess.close()


def test_sharding_does_not_change_gpu_results(rt):
    """Spilled execution equals unspilled execution (paper Section 2.3): k = 1, 2, 4 layers per shard give the
    same logits, loss and updated weights on the GPU, bit for bit (all reductions have a fixed order)."""
    H, R = rt
    outs = []
    for k in (1, 2, 4):
        cfg = SI.small_cfg(L=4, d=64, H=4, F=256, V=211, T=64, B=2, k=k, dtype="bf16")
        W = SI.make_weights(cfg, 9)
        tok, tgt = SI.make_batch(cfg, 10)
        sess = R.Session(R.arena_bytes_for([cfg], 3), max_slots=2)
        rec = sess.add_model(cfg, W, 1e-3)
        got = sess.train_step_manual(rec, tok, tgt)
        H.hydra_sync(sess.ctx)
        outs.append((got["logits"].copy(), got["loss"], {n: v.copy() for n, v in sess.unpack(rec, rec["master"]).items()}))
        sess.close()
    for o in outs[1:]:
        assert (o[0] == outs[0][0]).all() and o[1] == outs[0][1]
        for name in o[2]:
            assert (o[2][name] == outs[0][2][name]).all(), name


@pytest.mark.parametrize("nm,flags", [(2, 0), (3, 6), (4, 0)])   # 6 = checkpoint spilling + poisoned buffers
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_micro_batches_equal_one_large_minibatch(rt, nm, flags, dtype):
    """A minibatch run as nm micro-batches per shard visit (gradients summed while the shard is resident) equals
    the oracle's single step on all nm*B samples: loss over all valid targets, every gradient, weights after
    two steps.  Micro-batches carry different numbers of valid targets, so averaging per micro-batch would fail."""
    H, R = rt
    base = SI.small_cfg(L=4, d=64, H=4, F=256, V=211, T=72, B=2, k=2, dtype=dtype, lrs=[1e-4])
    big = dict(base, B=base["B"] * nm)
    cfg = dict(base, n_micro=nm)
    W = SI.make_weights(base, 77)
    batches = []
    for i in range(2):
        tok, tgt = SI.make_batch(big, 900 + i, zipf=(i == 1))
        tgt[: base["B"], 5:] = -1          # the first micro-batch has few valid targets
        batches.append((tok, tgt))
    refs, P, Mo, Vo = oracle_steps(big, W, 1e-4, batches)
    sess = R.Session(R.arena_bytes_for([cfg], 4, bool(flags & H.FLAG_CKPT_SPILL)), flags=flags, max_slots=3)
    rec = sess.add_model(cfg, W, 1e-4)
    ill, tol, M = {}, TOL[dtype], base["B"] * base["T"]
    for i, (tok, tgt) in enumerate(batches):
        got = sess.train_step_manual(rec, tok, tgt)
        H.hydra_sync(sess.ctx)
        assert_close(got["logits"], refs[i]["logits"][-M:], tol, "logits of the last micro-batch")
        assert abs(got["loss"] - refs[i]["loss"]) <= tol * abs(refs[i]["loss"])
        for name, g in refs[i]["grads"].items():
            assert_close(got["grads"][name], g, tol, f"grad {name}")
        update_ill(ill, refs[i]["grads"], dtype)
        after = {k: v.copy() for k, v in sess.unpack(rec, rec["master"]).items()}
        check_weights(after, refs[i]["after"], refs[0]["before"], ill, 1e-4, i + 1, dtype, f"step {i}: ")
    sess.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_scheduled_run_with_micro_batches(rt, dtype):
    """Two models, one with 3 micro-batches per visit and one with 1, through the scheduler on two lanes with
    three shard buffers; weights after two minibatches each against the oracle on the full minibatches."""
    H, R = rt
    base = SI.small_cfg(L=4, d=64, H=4, F=256, V=211, T=64, B=2, k=2, dtype=dtype, n_models=2, lrs=[1e-4, 3e-4])
    nms = [3, 1]
    cfgs = [dict(base, n_micro=nm) for nm in nms]
    bigs = [dict(base, B=base["B"] * nm) for nm in nms]
    Ws = [SI.make_weights(base, 50 + m) for m in range(2)]
    batches = [[SI.make_batch(bigs[m], 800 + 10 * m + i) for i in range(2)] for m in range(2)]
    fc, bc = SI.task_costs(base)
    sess = R.Session(R.arena_bytes_for(cfgs, 3, lanes=2), max_slots=3, lanes=2, flags=H.FLAG_POISON)
    recs = [sess.add_model(cfgs[m], Ws[m], base["lrs"][m]) for m in range(2)]
    sch = H.hydra_sched_create(sess.ctx, [r["id"] for r in recs], [2, 2], [list(fc) + list(bc)] * 2)
    toks = [np.stack([b[0] for b in batches[m]]) for m in range(2)]
    tgts = [np.stack([b[1] for b in batches[m]]) for m in range(2)]
    H.hydra_sched_run(sch, toks, tgts, sess.ctx)
    sess.flush()
    for m in range(2):
        refs, P, _, _ = oracle_steps(bigs[m], Ws[m], base["lrs"][m], batches[m])
        ill = {}
        for r in refs:
            update_ill(ill, r["grads"], dtype)
        assert abs(H.hydra_get_loss(sess.ctx, recs[m]["id"]) - refs[-1]["loss"]) <= TOL[dtype] * refs[-1]["loss"]
        check_weights(sess.unpack(recs[m], recs[m]["master"]), P, refs[0]["before"], ill, base["lrs"][m], 2, dtype,
                      f"model {m} ")
    H.hydra_sched_destroy(sch)
    sess.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_pilot_pass_measures_costs_and_leaves_the_model_untouched(rt, dtype):
    """Pilot pass (paper Section 2.2): per-task durations for the scheduler; nothing of the pass may survive - the
    host arrays stay bit-identical and the first real step still equals the oracle's step 1.  The scheduler then
    runs two models on the measured tables and its order equals the oracle's Sharded-LRTF on the same numbers."""
    H, R = rt
    cfg = SI.small_cfg(L=4, d=64, H=4, F=256, V=211, T=64, B=2, k=2, dtype=dtype, n_models=2, lrs=[1e-3, 3e-4])
    S, n = 2, 4
    Ws = [SI.make_weights(cfg, 60 + m) for m in range(2)]
    sess = R.Session(R.arena_bytes_for([cfg] * 2, 3), max_slots=3)
    recs = [sess.add_model(cfg, Ws[m], cfg["lrs"][m]) for m in range(2)]
    tables = []
    for m in range(2):
        before = [recs[m][k].copy() for k in ("master", "m", "v")]
        tok, tgt = SI.make_batch(cfg, 990 + m)
        costs = H.hydra_pilot_costs(sess.ctx, recs[m]["id"], tok, tgt, n)
        assert len(costs) == 2 * n and all(c > 0 for c in costs)
        # (no ordering between the measured durations is asserted: on a model this small a task is shorter than the
        # host's jitter in enqueueing it)
        assert max(costs) < 5_000_000_000
        for k, b in zip(("master", "m", "v"), before):
            assert (recs[m][k] == b).all()
        tables.append(costs)
    # scheduler on the measured tables: same decisions as the oracle
    nmb = [2, 1]
    chains = [SP.model_task_chain(cfg, nmb[m]) for m in range(2)]
    costs = [[tables[m][s if ph == SP.FWD else n + s] for s, ph in chains[m]] for m in range(2)]
    order = SP.sharded_lrtf(chains, costs)
    batches = [[SI.make_batch(cfg, 700 + 10 * m + i) for i in range(nmb[m])] for m in range(2)]
    sch = H.hydra_sched_create(sess.ctx, [r["id"] for r in recs], nmb, tables)
    toks = [np.stack([b[0] for b in batches[m]]) for m in range(2)]
    tgts = [np.stack([b[1] for b in batches[m]]) for m in range(2)]
    trace, done = H.hydra_sched_run(sch, toks, tgts, sess.ctx, trace_cap=256)
    sess.flush()
    per = 2 * n
    assert trace == [(m, chains[m][i][0], chains[m][i][1], i // per) for m, i in order]
    for m in range(2):
        refs, P, _, _ = oracle_steps(cfg, Ws[m], cfg["lrs"][m], batches[m])   # Adam step counter starts at 1
        ill = {}
        for r in refs:
            update_ill(ill, r["grads"], dtype)
        check_weights(sess.unpack(recs[m], recs[m]["master"]), P, refs[0]["before"], ill, cfg["lrs"][m], nmb[m], dtype,
                      f"model {m} ")
    H.hydra_sched_destroy(sch)
    sess.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_heterogeneous_models_in_one_job(rt, dtype):
    """Three models of different depth, width, batch, sequence length, shard size and micro-batch count in one
    scheduled run on two lanes with four shard buffers (paper Section 2.4: the scheduler exists for unequal
    models).  Order against the oracle's Sharded-LRTF (and it is not round-robin); weights against the oracle."""
    H, R = rt
    cfgs = [SI.small_cfg(L=4, d=64, H=4, F=256, V=211, T=64, B=2, k=2, dtype=dtype, lrs=[1e-4]),
            SI.small_cfg(L=2, d=128, H=4, F=512, V=300, T=72, B=1, k=1, dtype=dtype, lrs=[3e-4]),
            dict(SI.small_cfg(L=6, d=32, H=2, F=128, V=97, T=40, B=2, k=3, dtype=dtype, lrs=[1e-4]), n_micro=2)]
    bigs = [dict(c, B=c["B"] * c.get("n_micro", 1)) for c in cfgs]
    nmb = [1, 2, 2]
    n = len(cfgs)
    Ws = [SI.make_weights(cfgs[m], 70 + m) for m in range(n)]
    batches = [[SI.make_batch(bigs[m], 600 + 10 * m + i) for i in range(nmb[m])] for m in range(n)]
    tabs = [SI.task_costs(c) for c in cfgs]
    chains = [SP.model_task_chain(cfgs[m], nmb[m]) for m in range(n)]
    costs = [[(tabs[m][0] if ph == SP.FWD else tabs[m][1])[s] for s, ph in chains[m]] for m in range(n)]
    order = SP.sharded_lrtf(chains, costs)
    sess = R.Session(R.arena_bytes_for(cfgs, 4, lanes=2), max_slots=4, lanes=2, flags=H.FLAG_POISON)
    recs = [sess.add_model(cfgs[m], Ws[m], cfgs[m]["lrs"][0]) for m in range(n)]
    sch = H.hydra_sched_create(sess.ctx, [r["id"] for r in recs], nmb, [list(t[0]) + list(t[1]) for t in tabs])
    toks = [np.stack([b[0] for b in batches[m]]) for m in range(n)]
    tgts = [np.stack([b[1] for b in batches[m]]) for m in range(n)]
    trace, done = H.hydra_sched_run(sch, toks, tgts, sess.ctx, trace_cap=4096)
    sess.flush()
    want = []
    for m, i in order:
        per = 2 * (cfgs[m]["L"] // cfgs[m]["k"] + 2)
        want.append((m, chains[m][i][0], chains[m][i][1], i // per))
    assert trace == want
    assert [t[0] for t in trace[:n]] != list(range(n))            # not a round-robin start
    for m in range(n):
        refs, P, _, _ = oracle_steps(bigs[m], Ws[m], cfgs[m]["lrs"][0], batches[m])
        ill = {}
        for r in refs:
            update_ill(ill, r["grads"], dtype)
        assert abs(H.hydra_get_loss(sess.ctx, recs[m]["id"]) - refs[-1]["loss"]) <= TOL[dtype] * refs[-1]["loss"]
        check_weights(sess.unpack(recs[m], recs[m]["master"]), P, refs[0]["before"], ill, cfgs[m]["lrs"][0], nmb[m],
                      dtype, f"model {m} ")
    H.hydra_sched_destroy(sch)
    sess.close()


@pytest.mark.parametrize("mode", ["manual_spill", "resident", "scheduled_micro"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_tied_lm_head(rt, dtype, mode):
    """LM head tied to the token embedding (logits = z wte^T): the HEAD shard owns only the final LayerNorm and
    works on a copy of wte; the wte gradient is the head's part plus the lookup's part and wte is stepped once,
    at the EMBED shard's backward visit.  Three minibatches, so that the head's copy has to be refreshed after
    every update - with every shard spilled between visits, with all shards resident (the update then exists only
    on the device), and through the scheduler with micro-batches."""
    H, R = rt
    base = SI.small_cfg(L=2, d=64, H=2, F=128, V=301, T=40, B=2, k=1, dtype=dtype, lrs=[1e-4], tie=True)
    nm = 2 if mode == "scheduled_micro" else 1
    cfg = dict(base, n_micro=nm)
    big = dict(base, B=base["B"] * nm)
    W = SI.make_weights(base, 31)
    assert "w_lm" not in W
    batches = [SI.make_batch(big, 400 + i, zipf=(i == 1)) for i in range(3)]
    refs, P, Mo, Vo = oracle_steps(big, W, 1e-4, batches)
    sess = R.Session(R.arena_bytes_for([cfg], 4), max_slots=2 if mode == "manual_spill" else 4,
                     flags=H.FLAG_POISON if mode == "manual_spill" else 0)
    rec = sess.add_model(cfg, W, 1e-4)
    assert rec["layout"].n_params == SI.n_params(base)
    ill, tol, M = {}, TOL[dtype], base["B"] * base["T"]
    if mode == "scheduled_micro":
        fc, bc = SI.task_costs(base)
        sch = H.hydra_sched_create(sess.ctx, [rec["id"]], [3], [list(fc) + list(bc)])
        H.hydra_sched_run(sch, [np.stack([b[0] for b in batches])], [np.stack([b[1] for b in batches])], sess.ctx)
        sess.flush()
        H.hydra_sched_destroy(sch)
        for r in refs:
            update_ill(ill, r["grads"], dtype)
        assert abs(H.hydra_get_loss(sess.ctx, rec["id"]) - refs[-1]["loss"]) <= tol * refs[-1]["loss"]
        check_weights(sess.unpack(rec, rec["master"]), P, refs[0]["before"], ill, 1e-4, 3, dtype)
    else:
        for i, (tok, tgt) in enumerate(batches):
            got = sess.train_step_manual(rec, tok, tgt, spill=(mode == "manual_spill"))
            H.hydra_sync(sess.ctx)
            assert_close(got["logits"], refs[i]["logits"][-M:], tol, "logits")
            assert abs(got["loss"] - refs[i]["loss"]) <= tol * abs(refs[i]["loss"])
            for name, g in refs[i]["grads"].items():
                assert_close(got["grads"][name], g, tol, f"grad {name}")
            update_ill(ill, refs[i]["grads"], dtype)
            if mode == "resident":
                sess.flush()
            after = {k: v.copy() for k, v in sess.unpack(rec, rec["master"]).items()}
            check_weights(after, refs[i]["after"], refs[0]["before"], ill, 1e-4, i + 1, dtype, f"step {i}: ")
    sess.close()


@pytest.mark.parametrize("max_slots,lanes,nm", [(0, 2, 1), (3, 1, 1), (4, 2, 2)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_graph_replay_of_shard_visits(rt, dtype, max_slots, lanes, nm):
    """HYDRA_FLAG_GRAPHS: the kernel sequence of a block-shard visit is captured on its second run with a given
    shard buffer and replayed afterwards.  Five minibatches of two models, so every combination is run plainly,
    captured and replayed several times with the uncaptured work (loads, Adam, write-backs, head, embedding) and
    stream synchronisations in between; weights and loss against the oracle after the last one, and the result
    must be bit-identical to the same run without graphs.  With few buffers the shards move between buffers, which
    gives one graph per (shard, buffer) pair."""
    H, R = rt
    base = SI.small_cfg(L=4, d=64, H=4, F=256, V=211, T=64, B=2, k=2, dtype=dtype, n_models=2, lrs=[1e-4, 3e-4])
    cfg = dict(base, n_micro=nm)
    big = dict(base, B=base["B"] * nm)
    n, steps = 2, 5
    Ws = [SI.make_weights(base, 80 + m) for m in range(n)]
    batches = [[SI.make_batch(big, 500 + 10 * m + i) for i in range(steps)] for m in range(n)]
    fc, bc = SI.task_costs(base)
    results = []
    for flags in (H.FLAG_GRAPHS, 0):
        sess = R.Session(R.arena_bytes_for([cfg] * n, 12, lanes=lanes), max_slots=max_slots, lanes=lanes, flags=flags)
        recs = [sess.add_model(cfg, Ws[m], base["lrs"][m]) for m in range(n)]
        sch = H.hydra_sched_create(sess.ctx, [r["id"] for r in recs], [steps] * n, [list(fc) + list(bc)] * n)
        toks = [np.stack([b[0] for b in batches[m]]) for m in range(n)]
        tgts = [np.stack([b[1] for b in batches[m]]) for m in range(n)]
        H.hydra_sched_run(sch, toks, tgts, sess.ctx)
        sess.flush()
        st = H.hydra_get_stats(sess.ctx)
        if flags:
            assert st["n_graph_launches"] > 0
        else:
            assert st["n_graph_launches"] == 0
        results.append(([sess.unpack(recs[m], recs[m]["master"].copy()) for m in range(n)],
                        [H.hydra_get_loss(sess.ctx, recs[m]["id"]) for m in range(n)]))
        H.hydra_sched_destroy(sch)
        sess.close()
    (wg, lg), (we, le) = results
    assert lg == le
    for m in range(n):
        for name in wg[m]:
            assert (wg[m][name] == we[m][name]).all(), name       # graphs change nothing
        refs, P, _, _ = oracle_steps(big, Ws[m], base["lrs"][m], batches[m])
        ill = {}
        for r in refs:
            update_ill(ill, r["grads"], dtype)
        assert abs(lg[m] - refs[-1]["loss"]) <= TOL[dtype] * refs[-1]["loss"]
        check_weights(wg[m], P, refs[0]["before"], ill, base["lrs"][m], steps, dtype, f"model {m} ")


def test_overlap_trace_of_a_spilled_run(rt):
    """HYDRA_FLAG_OVERLAP: the event pairs around promotes, write-backs and shard tasks of a spilled two-model run
    give interval unions that are consistent with each other and with the byte counters; without the flag the call
    reports a state error.  The traced run's weights equal those of an untraced run bit for bit."""
    H, R = rt
    cfg = SI.small_cfg(L=4, d=64, H=4, F=256, V=211, T=64, B=2, k=1, dtype="bf16", n_models=2, lrs=[1e-4, 3e-4])
    n, steps = 2, 3
    Ws = [SI.make_weights(cfg, 60 + m) for m in range(n)]
    batches = [[SI.make_batch(cfg, 900 + 10 * m + i) for i in range(steps)] for m in range(n)]
    fc, bc = SI.task_costs(cfg)
    finals = []
    for flags in (H.FLAG_OVERLAP, 0):
        sess = R.Session(R.arena_bytes_for([cfg] * n, 3, lanes=2), max_slots=3, lanes=2, flags=flags)
        recs = [sess.add_model(cfg, Ws[m], cfg["lrs"][m]) for m in range(n)]
        sch = H.hydra_sched_create(sess.ctx, [r["id"] for r in recs], [steps] * n, [list(fc) + list(bc)] * n)
        toks = [np.stack([b[0] for b in batches[m]]) for m in range(n)]
        tgts = [np.stack([b[1] for b in batches[m]]) for m in range(n)]
        st0 = H.hydra_get_stats(sess.ctx)
        H.hydra_sched_run(sch, toks, tgts, sess.ctx)
        if flags:
            o = H.hydra_overlap_stats(sess.ctx)
            st1 = H.hydra_get_stats(sess.ctx)
            assert o["n_intervals"] > 0 and o["wall_ms"] > 0
            assert o["bytes_h2d"] == st1["bytes_h2d"] - st0["bytes_h2d"]
            assert o["bytes_d2h"] == st1["bytes_d2h"] - st0["bytes_d2h"]
            eps = 1e-6
            assert 0 < o["compute_ms"] <= o["wall_ms"] + eps
            assert max(o["h2d_ms"], o["d2h_ms"]) <= o["transfer_ms"] + eps <= o["h2d_ms"] + o["d2h_ms"] + 2 * eps
            assert 0 <= o["hidden_ms"] <= min(o["transfer_ms"], o["compute_ms"]) + eps
            assert o["transfer_ms"] <= o["wall_ms"] + eps
            H.hydra_overlap_reset(sess.ctx)
            assert H.hydra_overlap_stats(sess.ctx)["n_intervals"] == 0
        else:
            with pytest.raises(H.HydraError) as ei:
                H.hydra_overlap_stats(sess.ctx)
            assert ei.value.code == H.E_STATE
        sess.flush()
        finals.append([recs[m]["master"].copy() for m in range(n)])
        H.hydra_sched_destroy(sch)
        sess.close()
    for a, b in zip(*finals):
        assert np.isfinite(a).all() and (a == b).all()
