"""CPU oracle: forward, backward and Adam of a GPT-2-style decoder in plain numpy.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module;
it exists so that the HIP library can be checked against an independent, slow,
obviously-correct implementation.  It shares no code with the HIP path.

What is computed.  The paper's method (spilled, shard-by-shard execution with
checkpoints at shard boundaries and recomputation in backward, Section 2.3) is
stated to be mathematically the same as ordinary training of the model, so the
defining computation is plain training: forward -> mean next-token
cross-entropy -> backward -> Adam.  The paper trains "HuggingFace GPT-2"
(Section 3) and gives none of the decoder's formulas; the readings taken here
(all from the published GPT-2 architecture and textbook definitions):

  * pre-LayerNorm blocks; LayerNorm with biased variance and eps = 1e-5
  * one fused QKV projection, heads = contiguous column groups of width d/H
  * scores scaled by 1/sqrt(d/H); causal mask; masked probabilities exactly 0
  * GELU in its tanh form
  * biases on the four linears of a block, none on the LM head
  * untied LM head W_lm[d, V]; learned positions wpe[T, d]; no dropout
  * loss = mean over positions whose target is >= 0
  * Adam (beta1 .9, beta2 .999, eps 1e-8), no weight decay, constant lr,
    bias corrections 1 - beta^t evaluated in double

Every routine works in the dtype of its inputs (float32 or float64): the
float64 instance is the reference for parity and finite differences, the
float32 instance is what is timed as the CPU baseline.  No blocking, fusion or
reordering: each step is the formula written out, numpy matmul being the only
library primitive.

Pins (tests/, run without a GPU): central finite differences of the loss for
every parameter tensor; an independent autograd build of the same network from
torch.nn.functional primitives and torch.optim.Adam; closed forms (loss = ln V
for zero logits, first Adam step = -lr*g/(|g|+eps)); invariants (softmax rows
sum to 1, masked entries exactly 0, causality, identity block when the output
projections are zero); sharded == unsharded bit for bit.
"""
from __future__ import annotations

import math

import numpy as np

LN_EPS = 1e-5
GELU_C = 0.044715


# --------------------------------------------------------------------------
# elementary operations, forward and backward
# --------------------------------------------------------------------------

def layernorm_fwd(x, gamma, beta):
    """Row-wise LayerNorm over the last axis.  Returns (y, cache)."""
    R = x.dtype.type
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    rstd = R(1.0) / np.sqrt(var + R(LN_EPS))
    xhat = xc * rstd
    return xhat * gamma + beta, (xhat, rstd)


def layernorm_bwd(dy, gamma, cache):
    """dx, dgamma, dbeta for y = xhat*gamma + beta."""
    xhat, rstd = cache
    dgamma = (dy * xhat).sum(axis=0)
    dbeta = dy.sum(axis=0)
    dxhat = dy * gamma
    m1 = dxhat.mean(axis=-1, keepdims=True)
    m2 = (dxhat * xhat).mean(axis=-1, keepdims=True)
    dx = rstd * (dxhat - m1 - xhat * m2)
    return dx, dgamma, dbeta


def linear_fwd(x, W, b=None):
    y = x @ W
    if b is not None:
        y = y + b
    return y


def linear_bwd(dy, x, W, has_bias=True):
    dx = dy @ W.T
    dW = x.T @ dy
    db = dy.sum(axis=0) if has_bias else None
    return dx, dW, db


def gelu_fwd(u):
    R = u.dtype.type
    c = R(math.sqrt(2.0 / math.pi))
    tau = np.tanh(c * (u + R(GELU_C) * u * u * u))
    return R(0.5) * u * (R(1.0) + tau)


def gelu_bwd(dg, u):
    R = u.dtype.type
    c = R(math.sqrt(2.0 / math.pi))
    tau = np.tanh(c * (u + R(GELU_C) * u * u * u))
    dtau = (R(1.0) - tau * tau) * c * (R(1.0) + R(3.0 * GELU_C) * u * u)
    return dg * (R(0.5) * (R(1.0) + tau) + R(0.5) * u * dtau)


def _split_heads(z, B, T, H):
    d = z.shape[-1]
    return z.reshape(B, T, H, d // H).transpose(0, 2, 1, 3)   # [B,H,T,dh]


def _merge_heads(z):
    B, H, T, dh = z.shape
    return z.transpose(0, 2, 1, 3).reshape(B * T, H * dh)


def attention_fwd(qkv, B, T, H):
    """Causal multi-head self-attention on a fused [M, 3d] projection.
    Returns (o [M, d], cache)."""
    R = qkv.dtype.type
    d = qkv.shape[-1] // 3
    dh = d // H
    q = _split_heads(qkv[:, 0:d], B, T, H)
    k = _split_heads(qkv[:, d:2 * d], B, T, H)
    v = _split_heads(qkv[:, 2 * d:3 * d], B, T, H)
    scale = R(1.0 / math.sqrt(dh))
    s = (q @ k.transpose(0, 1, 3, 2)) * scale                 # [B,H,T,T]
    allowed = np.tril(np.ones((T, T), dtype=bool))            # j <= i
    s = np.where(allowed, s, R(-np.inf))
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    e = np.where(allowed, e, R(0.0))
    p = e / e.sum(axis=-1, keepdims=True)
    o = _merge_heads(p @ v)
    return o, (q, k, v, p, scale)


def attention_bwd(do, cache, B, T, H):
    """Gradient w.r.t. the fused qkv input, [M, 3d]."""
    q, k, v, p, scale = cache
    do_h = _split_heads(do, B, T, H)                          # [B,H,T,dh]
    dv = p.transpose(0, 1, 3, 2) @ do_h
    dp = do_h @ v.transpose(0, 1, 3, 2)
    ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))      # zero where p is zero
    dq = (ds @ k) * scale
    dk = (ds.transpose(0, 1, 3, 2) @ q) * scale
    return np.concatenate([_merge_heads(dq), _merge_heads(dk), _merge_heads(dv)], axis=1)


def embed_fwd(tokens, wte, wpe):
    B, T = tokens.shape
    x = wte[tokens.reshape(-1)] + np.tile(wpe[:T], (B, 1))
    return x


def embed_bwd(dx, tokens, V):
    B, T = tokens.shape
    d = dx.shape[-1]
    dwte = np.zeros((V, d), dx.dtype)
    # unbuffered, in index order: sample-major, position-minor
    np.add.at(dwte, tokens.reshape(-1), dx)
    dwpe = dx.reshape(B, T, d).sum(axis=0)
    return dwte, dwpe


def cross_entropy(logits, targets):
    """Mean negative log-likelihood over positions with target >= 0.
    Returns (loss as python float, dlogits)."""
    R = logits.dtype.type
    tgt = targets.reshape(-1)
    valid = tgt >= 0
    n = int(valid.sum())
    zmax = logits.max(axis=-1, keepdims=True)
    e = np.exp(logits - zmax)
    se = e.sum(axis=-1, keepdims=True)
    lse = np.log(se) + zmax                                   # [M,1]
    rows = np.nonzero(valid)[0]
    nll = lse[rows, 0] - logits[rows, tgt[rows]]
    loss = float(np.sum(nll.astype(np.float64)) / n)
    dlogits = e / se
    dlogits[rows, tgt[rows]] -= R(1.0)
    dlogits[~valid] = R(0.0)
    dlogits *= R(1.0 / n)
    return loss, dlogits


# --------------------------------------------------------------------------
# the three kinds of shard: embedding, run of blocks, head
# --------------------------------------------------------------------------

BLOCK_TENSORS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                 "ln2_g", "ln2_b", "w_fc", "b_fc", "w_proj", "b_proj")


def block_fwd(P, l, x, B, T, H):
    """One pre-LN transformer block.  Returns (x_out, cache)."""
    p = lambda n: P[f"h{l}.{n}"]
    a, ln1 = layernorm_fwd(x, p("ln1_g"), p("ln1_b"))
    qkv = linear_fwd(a, p("w_qkv"), p("b_qkv"))
    o, att = attention_fwd(qkv, B, T, H)
    x1 = x + linear_fwd(o, p("w_o"), p("b_o"))
    c, ln2 = layernorm_fwd(x1, p("ln2_g"), p("ln2_b"))
    u = linear_fwd(c, p("w_fc"), p("b_fc"))
    g = gelu_fwd(u)
    x2 = x1 + linear_fwd(g, p("w_proj"), p("b_proj"))
    return x2, (a, ln1, att, o, c, ln2, u, g)


def block_bwd(P, l, dx2, cache, B, T, H):
    """Returns (dx, grads dict for this block)."""
    p = lambda n: P[f"h{l}.{n}"]
    a, ln1, att, o, c, ln2, u, g = cache
    G = {}
    dg, G[f"h{l}.w_proj"], G[f"h{l}.b_proj"] = linear_bwd(dx2, g, p("w_proj"))
    du = gelu_bwd(dg, u)
    dc, G[f"h{l}.w_fc"], G[f"h{l}.b_fc"] = linear_bwd(du, c, p("w_fc"))
    dx1_ln, G[f"h{l}.ln2_g"], G[f"h{l}.ln2_b"] = layernorm_bwd(dc, p("ln2_g"), ln2)
    dx1 = dx2 + dx1_ln
    do, G[f"h{l}.w_o"], G[f"h{l}.b_o"] = linear_bwd(dx1, o, p("w_o"))
    dqkv = attention_bwd(do, att, B, T, H)
    da, G[f"h{l}.w_qkv"], G[f"h{l}.b_qkv"] = linear_bwd(dqkv, a, p("w_qkv"))
    dx_ln, G[f"h{l}.ln1_g"], G[f"h{l}.ln1_b"] = layernorm_bwd(da, p("ln1_g"), ln1)
    return dx1 + dx_ln, G


def head_fwd(P, x):
    """Final LayerNorm and logits.  A model without "w_lm" ties the LM head to the
    token embedding: logits = z @ wte^T."""
    z, lnf = layernorm_fwd(x, P["lnf_g"], P["lnf_b"])
    logits = linear_fwd(z, P["w_lm"] if "w_lm" in P else P["wte"].T)
    return logits, (z, lnf)


def head_bwd(P, dlogits, cache):
    """Tied head: the gradient of wte through the logits comes back as
    G["wte_head"] ([V, d]); the caller adds the embedding lookup's part."""
    z, lnf = cache
    G = {}
    if "w_lm" in P:
        dz, G["w_lm"], _ = linear_bwd(dlogits, z, P["w_lm"], has_bias=False)
    else:
        dz, gw, _ = linear_bwd(dlogits, z, P["wte"].T, has_bias=False)
        G["wte_head"] = np.ascontiguousarray(gw.T)
    dx, G["lnf_g"], G["lnf_b"] = layernorm_bwd(dz, P["lnf_g"], lnf)
    return dx, G


# --------------------------------------------------------------------------
# Adam
# --------------------------------------------------------------------------

def adam_update(w, m, v, g, t, lr, beta1=0.9, beta2=0.999, eps=1e-8):
    """One Adam step on one tensor; returns new (w, m, v).  t counts from 1."""
    R = w.dtype.type
    m = R(beta1) * m + R(1.0 - beta1) * g
    v = R(beta2) * v + R(1.0 - beta2) * (g * g)
    c1 = R(1.0 - beta1 ** t)          # python floats are doubles
    c2 = R(1.0 - beta2 ** t)
    mhat = m / c1
    vhat = v / c2
    w = w - R(lr) * mhat / (np.sqrt(vhat) + R(eps))
    return w, m, v


# --------------------------------------------------------------------------
# plain (unsharded) training step: the definition
# --------------------------------------------------------------------------

def cast_params(P, dtype):
    return {k: np.asarray(a, dtype=dtype) for k, a in P.items()}


def zeros_like_params(P):
    return {k: np.zeros_like(a) for k, a in P.items()}


def forward_backward(P, tokens, targets, cfg):
    """Full forward and backward without any sharding.
    Returns dict(logits, loss, grads)."""
    B, T = tokens.shape
    H, L, V = cfg["H"], cfg["L"], cfg["V"]
    x = embed_fwd(tokens, P["wte"], P["wpe"])
    caches = []
    for l in range(L):
        x, c = block_fwd(P, l, x, B, T, H)
        caches.append(c)
    logits, hc = head_fwd(P, x)
    loss, dlogits = cross_entropy(logits, targets)
    G = {}
    dx, g = head_bwd(P, dlogits, hc)
    G.update(g)
    for l in reversed(range(L)):
        dx, g = block_bwd(P, l, dx, caches[l], B, T, H)
        G.update(g)
    G["wte"], G["wpe"] = embed_bwd(dx, tokens, V)
    if "wte_head" in G:
        G["wte"] = G.pop("wte_head") + G["wte"]
    return dict(logits=logits, loss=loss, grads=G)


def train_step(P, Mo, Vo, tokens, targets, cfg, lr, t):
    """One plain training step.  Updates P, Mo, Vo (dicts) in place and
    returns dict(logits, loss, grads)."""
    out = forward_backward(P, tokens, targets, cfg)
    for name in P:
        P[name], Mo[name], Vo[name] = adam_update(P[name], Mo[name], Vo[name],
                                                  out["grads"][name], t, lr)
    return out
