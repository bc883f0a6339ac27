"""Pins for the CPU oracle: everything here checks oracle/ against something
other than itself - finite differences, closed forms, invariants, and an
independent autograd build from torch.nn.functional primitives."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as TF

import synth_inputs as SI
from oracle import decoder as D
from oracle import spilled as SP


def _setup(dtype=np.float64, **kw):
    cfg = SI.small_cfg(**kw)
    P = D.cast_params(SI.make_weights(cfg, cfg["wseed"]), dtype)
    tok, tgt = SI.make_batch(cfg, cfg["dseed"])
    return cfg, P, tok, tgt


# ---------------------------------------------------------------- P-FD
@pytest.mark.parametrize("tie", [False, True])
def test_finite_differences_every_tensor(tie):
    cfg, P, tok, tgt = _setup(tie=tie)
    assert ("w_lm" in P) != tie
    out = D.forward_backward(P, tok, tgt, cfg)
    rng = np.random.default_rng(0)
    h = 1e-5
    worst = 0.0
    for name, shape, _ in SI.tensor_shapes(cfg):
        a = P[name]
        flat = a.reshape(-1)
        n = flat.size
        idx = np.arange(n) if n <= 48 else rng.choice(n, 24, replace=False)
        if name == "wte":   # make sure rows that are actually used get probed
            used = np.unique(tok)[:6]
            idx = np.concatenate([idx, used * cfg["d"] + 1])
        for i in idx:
            old = flat[i]
            flat[i] = old + h
            lp = D.forward_backward(P, tok, tgt, cfg)["loss"]
            flat[i] = old - h
            lm = D.forward_backward(P, tok, tgt, cfg)["loss"]
            flat[i] = old
            fd = (lp - lm) / (2 * h)
            an = out["grads"][name].reshape(-1)[i]
            err = abs(fd - an) / max(1e-6, abs(fd) + abs(an))
            worst = max(worst, err)
            assert err < 2e-6 or abs(fd - an) < 1e-9, (name, i, fd, an)
    assert worst < 1e-4


# ---------------------------------------------------------------- P-lib
def _torch_model(Pt, tok, tgt, cfg):
    B, T = tok.shape
    d, H, L = cfg["d"], cfg["H"], cfg["L"]
    dh = d // H
    tk = torch.as_tensor(tok, dtype=torch.long)
    x = Pt["wte"][tk] + Pt["wpe"][None, :T]
    for l in range(L):
        g = lambda n: Pt[f"h{l}.{n}"]
        a = TF.layer_norm(x, (d,), g("ln1_g"), g("ln1_b"), eps=1e-5)
        qkv = a @ g("w_qkv") + g("b_qkv")
        q, k, v = qkv.split(d, dim=-1)
        sh = lambda z: z.view(B, T, H, dh).transpose(1, 2)
        o = TF.scaled_dot_product_attention(sh(q), sh(k), sh(v), is_causal=True)
        o = o.transpose(1, 2).reshape(B, T, d)
        x = x + o @ g("w_o") + g("b_o")
        c = TF.layer_norm(x, (d,), g("ln2_g"), g("ln2_b"), eps=1e-5)
        u = c @ g("w_fc") + g("b_fc")
        x = x + TF.gelu(u, approximate="tanh") @ g("w_proj") + g("b_proj")
    z = TF.layer_norm(x, (d,), Pt["lnf_g"], Pt["lnf_b"], eps=1e-5)
    logits = z @ (Pt["w_lm"] if "w_lm" in Pt else Pt["wte"].T)
    loss = TF.cross_entropy(logits.view(B * T, -1),
                            torch.as_tensor(tgt, dtype=torch.long).view(-1), ignore_index=-1)
    return logits, loss


@pytest.mark.parametrize("kw", [dict(), dict(L=3, d=24, H=3, F=40, V=50, T=12, B=3),
                                dict(L=2, d=16, H=2, F=32, V=40, T=8, B=2, tie=True)])
def test_against_torch_autograd_and_adam(kw):
    cfg, P, tok, tgt = _setup(**kw)
    Pt = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in P.items()}
    opt = torch.optim.Adam(list(Pt.values()), lr=1e-3, betas=(0.9, 0.999), eps=1e-8)
    Mo, Vo = D.zeros_like_params(P), D.zeros_like_params(P)
    for t in (1, 2, 3):
        tok, tgt = SI.make_batch(cfg, cfg["dseed"] + t)
        opt.zero_grad()
        logits_t, loss_t = _torch_model(Pt, tok, tgt, cfg)
        loss_t.backward()
        grads_t = {k: v.grad.detach().numpy().copy() for k, v in Pt.items()}
        opt.step()
        out = D.train_step(P, Mo, Vo, tok, tgt, cfg, 1e-3, t)
        np.testing.assert_allclose(out["logits"], logits_t.detach().numpy().reshape(out["logits"].shape),
                                   rtol=1e-10, atol=1e-12)
        assert abs(out["loss"] - loss_t.item()) < 1e-12
        for k in P:
            np.testing.assert_allclose(out["grads"][k], grads_t[k], rtol=1e-8, atol=1e-13, err_msg=k)
            np.testing.assert_allclose(P[k], Pt[k].detach().numpy(), rtol=1e-9, atol=1e-13, err_msg=k)


def test_gelu_is_tanh_form_not_erf():
    u = np.linspace(-4, 4, 801)
    ours = D.gelu_fwd(u)
    tanh_t = TF.gelu(torch.tensor(u), approximate="tanh").numpy()
    erf_t = TF.gelu(torch.tensor(u)).numpy()
    assert np.abs(ours - tanh_t).max() < 1e-14
    assert np.abs(ours - erf_t).max() > 1e-4      # the two forms are distinguishable


# ---------------------------------------------------------------- P-softmax / P-T1
@pytest.mark.parametrize("dtype,tol", [(np.float32, 1e-6), (np.float64, 1e-14)])
def test_softmax_rows_and_mask(dtype, tol):
    rng = np.random.default_rng(3)
    B, T, H, d = 2, 9, 3, 12
    qkv = rng.standard_normal((B * T, 3 * d)).astype(dtype) * 3
    o, (q, k, v, p, _) = D.attention_fwd(qkv, B, T, H)
    assert p.dtype == dtype
    assert np.abs(p.sum(-1) - 1).max() <= tol
    assert (p >= 0).all()
    iu = np.triu_indices(T, 1)
    assert (p[:, :, iu[0], iu[1]] == 0.0).all()
    assert (p[:, :, 0, 0] == 1.0).all()


def test_attention_T1_returns_v_and_head_extremes():
    rng = np.random.default_rng(4)
    d = 8
    for H in (1, 2, d):
        qkv = rng.standard_normal((3, 3 * d))
        o, _ = D.attention_fwd(qkv, 3, 1, H)
        assert (o == qkv[:, 2 * d:]).all()


def test_attention_matches_bruteforce_loops():
    rng = np.random.default_rng(5)
    B, T, H, d = 2, 5, 2, 6
    dh = d // H
    qkv = rng.standard_normal((B * T, 3 * d))
    o, _ = D.attention_fwd(qkv, B, T, H)
    ref = np.zeros((B * T, d))
    for b in range(B):
        for h in range(H):
            for i in range(T):
                qi = qkv[b * T + i, h * dh:(h + 1) * dh]
                sc = [qi @ qkv[b * T + j, d + h * dh:d + (h + 1) * dh] / math.sqrt(dh) for j in range(i + 1)]
                w = np.exp(np.array(sc) - max(sc))
                w /= w.sum()
                for j in range(i + 1):
                    ref[b * T + i, h * dh:(h + 1) * dh] += w[j] * qkv[b * T + j, 2 * d + h * dh:2 * d + (h + 1) * dh]
    np.testing.assert_allclose(o, ref, rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- P-causal
def test_causality_and_sample_independence_bitwise():
    cfg, P, tok, tgt = _setup(dtype=np.float32, T=10)
    base = D.forward_backward(P, tok, tgt, cfg)["logits"].reshape(cfg["B"], cfg["T"], -1)
    t0 = 6
    tok2 = tok.copy()
    tok2[1, t0] = (tok2[1, t0] + 1) % cfg["V"]
    new = D.forward_backward(P, tok2, tgt, cfg)["logits"].reshape(cfg["B"], cfg["T"], -1)
    assert (new[0] == base[0]).all()
    assert (new[1, :t0] == base[1, :t0]).all()
    assert (new[1, t0] != base[1, t0]).any()


# ---------------------------------------------------------------- P-ident
def test_block_is_identity_when_output_projections_vanish():
    cfg, P, tok, tgt = _setup(dtype=np.float32)
    for n in ("w_o", "b_o", "w_proj", "b_proj"):
        P[f"h0.{n}"][...] = 0
    x = np.random.default_rng(1).standard_normal((cfg["B"] * cfg["T"], cfg["d"])).astype(np.float32)
    y, _ = D.block_fwd(P, 0, x, cfg["B"], cfg["T"], cfg["H"])
    assert (y == x).all()


# ---------------------------------------------------------------- P-LN
def test_layernorm_statistics_and_backward_row_sum():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((7, 64)) * 3 + 5
    y, cache = D.layernorm_fwd(x, np.ones(64), np.zeros(64))
    assert np.abs(y.mean(-1)).max() < 1e-14
    var = x.var(-1)
    np.testing.assert_allclose(y.var(-1), var / (var + 1e-5), rtol=1e-12)
    ref = TF.layer_norm(torch.tensor(x), (64,), eps=1e-5).numpy()
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-13)
    dx, dg, db = D.layernorm_bwd(rng.standard_normal((7, 64)), rng.standard_normal(64), cache)
    assert np.abs(dx.sum(-1)).max() < 1e-13


# ---------------------------------------------------------------- P-CE
@pytest.mark.parametrize("V", [512, 50257, 50400])
def test_cross_entropy_closed_form_zero_logits(V):
    M = 6
    tgt = np.array([0, V - 1, -1, 5, 7, -1]).reshape(1, M)
    loss, dl = D.cross_entropy(np.zeros((M, V)), tgt)
    assert abs(loss - math.log(V)) < 1e-12
    golden = {512: 6.2383, 50257: 10.8249, 50400: 10.8277}[V]    # ln V to 4 decimals
    assert abs(loss - golden) < 6e-5
    assert (dl[[2, 5]] == 0).all()
    assert np.abs(dl[[0, 1, 3, 4]].sum(-1)).max() < 1e-15
    assert abs(dl[0, 0] - (1.0 / V - 1) / 4) < 1e-15


def test_loss_near_lnV_at_init():
    cfg, P, tok, tgt = _setup(dtype=np.float32, V=512, d=32, F=128)
    out = D.forward_backward(P, tok, tgt, cfg)
    assert abs(out["loss"] - math.log(512)) < 5e-2


# ---------------------------------------------------------------- P-embed
def test_embedding_indexing_and_absent_rows():
    cfg, P, tok, tgt = _setup(dtype=np.float32, V=64)
    x0 = D.embed_fwd(tok, P["wte"], P["wpe"])
    for b in range(cfg["B"]):
        for t in range(cfg["T"]):
            assert (x0[b * cfg["T"] + t] == P["wte"][tok[b, t]] + P["wpe"][t]).all()
    old = {k: v.copy() for k, v in P.items()}
    Mo, Vo = D.zeros_like_params(P), D.zeros_like_params(P)
    out = D.train_step(P, Mo, Vo, tok, tgt, cfg, 1e-3, 1)
    absent = np.setdiff1d(np.arange(cfg["V"]), np.unique(tok))
    assert absent.size > 0
    assert (out["grads"]["wte"][absent] == 0).all()
    assert (P["wte"][absent] == old["wte"][absent]).all()
    assert (Mo["wte"][absent] == 0).all() and (Vo["wte"][absent] == 0).all()
    present = np.unique(tok)
    assert (P["wte"][present] != old["wte"][present]).any()
    # repeated ids accumulate
    dx = np.arange(2 * 3 * 4, dtype=np.float64).reshape(6, 4)
    tk = np.array([[1, 1, 2], [1, 0, 2]])
    dwte, dwpe = D.embed_bwd(dx, tk, 4)
    assert (dwte[1] == dx[0] + dx[1] + dx[3]).all() and (dwte[3] == 0).all()
    assert (dwpe == dx[:3] + dx[3:]).all()


# ---------------------------------------------------------------- P-Adam
def test_adam_closed_forms():
    rng = np.random.default_rng(9)
    w = rng.standard_normal(100).astype(np.float32)
    g = rng.standard_normal(100).astype(np.float32)
    g[:5] = 0
    z = np.zeros_like(w)
    w1, m1, v1 = D.adam_update(w, z, z, g, 1, 1e-3)
    expect = -1e-3 * g.astype(np.float64) / (np.abs(g.astype(np.float64)) + 1e-8)
    np.testing.assert_allclose((w1 - w)[5:], expect[5:], rtol=2e-3)     # fp32 rounding of w + dw
    assert (w1[:5] == w[:5]).all()
    w0, _, _ = D.adam_update(w, z, z, g, 1, 0.0)
    assert (w0 == w).all()
    # two steps by hand on a scalar, in double
    wd, md, vd = 0.5, 0.0, 0.0
    W, Mm, Vv = np.array([0.5]), np.zeros(1), np.zeros(1)
    for t, gg in ((1, 0.3), (2, -0.7)):
        md = 0.9 * md + 0.1 * gg
        vd = 0.999 * vd + 0.001 * gg * gg
        wd -= 1e-2 * (md / (1 - 0.9 ** t)) / (math.sqrt(vd / (1 - 0.999 ** t)) + 1e-8)
        W, Mm, Vv = D.adam_update(W, Mm, Vv, np.array([gg]), t, 1e-2)
    assert abs(W[0] - wd) < 1e-15


# ---------------------------------------------------------------- P-shard / P-models
@pytest.mark.parametrize("tie", [False, True])
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("k", [1, 2, 4])
def test_sharded_equals_unsharded_bitwise(dtype, k, tie):
    cfg = SI.small_cfg(L=4, k=k, tie=tie)
    W = SI.make_weights(cfg, 11)
    P = D.cast_params(W, dtype)
    Mo, Vo = D.zeros_like_params(P), D.zeros_like_params(P)
    sm = SP.SpilledModel(cfg, W, 1e-3, dtype)
    chain = SP.model_task_chain(cfg, 1)
    for step in (1, 2):
        tok, tgt = SI.make_batch(cfg, 100 + step)
        ref = D.train_step(P, Mo, Vo, tok, tgt, cfg, 1e-3, step)
        sm.set_batch(tok, tgt)
        for s, ph in chain:
            sm.run_task(s, ph)
        assert sm.loss == ref["loss"]
        assert (sm.logits == ref["logits"]).all()
        for name in P:
            assert (sm.grads[name] == ref["grads"][name]).all(), name
            assert (sm.P[name] == P[name]).all(), name
            assert (sm.Mo[name] == Mo[name]).all() and (sm.Vo[name] == Vo[name]).all()


def test_interleaved_models_equal_models_alone_bitwise():
    cfg = SI.small_cfg(L=2, k=1, n_models=3, lrs=[1e-3, 3e-4, 1e-4])
    Ws = [SI.make_weights(cfg, 20 + m) for m in range(3)]
    nmb = [2, 1, 2]
    batches = [[SI.make_batch(cfg, 300 + 10 * m + i) for i in range(nmb[m])] for m in range(3)]
    chains = [SP.model_task_chain(cfg, nmb[m]) for m in range(3)]
    fc, bc = SI.task_costs(cfg)
    costs = [[(fc if ph == SP.FWD else bc)[s] for s, ph in ch] for ch in chains]
    order = SP.sharded_lrtf(chains, costs)
    inter = [SP.SpilledModel(cfg, Ws[m], cfg["lrs"][m], np.float32) for m in range(3)]
    SP.run_interleaved(inter, batches, order, chains)
    for m in range(3):
        P = D.cast_params(Ws[m], np.float32)
        Mo, Vo = D.zeros_like_params(P), D.zeros_like_params(P)
        for i in range(nmb[m]):
            D.train_step(P, Mo, Vo, *batches[m][i], cfg, cfg["lrs"][m], i + 1)
        for name in P:
            assert (inter[m].P[name] == P[name]).all(), (m, name)
    # same init, different lr: the models differ after one step only through Adam
    a = SP.SpilledModel(cfg, Ws[0], 1e-3, np.float32)
    b = SP.SpilledModel(cfg, Ws[0], 1e-4, np.float32)
    for mm in (a, b):
        mm.set_batch(*batches[0][0])
        for s, ph in SP.model_task_chain(cfg, 1):
            mm.run_task(s, ph)
    assert a.loss == b.loss
    assert all((a.grads[n] == b.grads[n]).all() for n in a.grads)
    assert any((a.P[n] != b.P[n]).any() for n in a.P)


def test_tied_head_gradient_is_the_sum_of_the_two_untied_gradients():
    """Tying the LM head to the token embedding (logits = z wte^T): same logits and loss as an untied model whose
    head matrix happens to equal wte^T, and the gradient of wte is the embedding part plus the transposed head
    part of that untied model."""
    cfg_t = SI.small_cfg(L=2, d=16, H=2, F=32, V=40, T=8, B=2, tie=True)
    cfg_u = dict(cfg_t, tie=False)
    Pt = D.cast_params(SI.make_weights(cfg_t, 5), np.float64)
    Pu = dict(Pt)
    Pu["w_lm"] = np.ascontiguousarray(Pt["wte"].T)
    tok, tgt = SI.make_batch(cfg_t, 6)
    ot = D.forward_backward(Pt, tok, tgt, cfg_t)
    ou = D.forward_backward(Pu, tok, tgt, cfg_u)
    assert np.array_equal(ot["logits"], ou["logits"]) and ot["loss"] == ou["loss"]
    np.testing.assert_allclose(ot["grads"]["wte"], ou["grads"]["wte"] + ou["grads"]["w_lm"].T, rtol=1e-12, atol=1e-15)
    for name in ot["grads"]:
        if name != "wte":
            np.testing.assert_allclose(ot["grads"][name], ou["grads"][name], rtol=1e-12, atol=1e-15, err_msg=name)
    assert SI.n_params(cfg_u) - SI.n_params(cfg_t) == cfg_t["d"] * cfg_t["V"]
