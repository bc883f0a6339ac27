"""Kernel-level parity on the GPU: each exported hydra_op_* is compared with
the oracle's routine for the same operation on seeded inputs whose sizes span
several tiles and leave ragged tails."""
import math

import numpy as np
import pytest

from oracle import decoder as D
from tests.parity_utils import assert_close, bf16_round

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def H():
    from paper_2110_08633_amd import hydra
    return hydra


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(dtype) if dtype is not None else t


def pad_cols(a, ld):
    out = np.zeros((a.shape[0], ld), a.dtype)
    out[:, :a.shape[1]] = a
    return out


GEMM_SHAPES = [(128, 128, 64), (200, 136, 72), (257, 72, 520), (64, 1001, 136), (520, 264, 200), (8, 8, 8)]


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 1), (1, 0)])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_all_layouts(H, dtype, ta, tb, M, N, K):
    rng = np.random.default_rng(M * 7 + N * 3 + K + ta * 2 + tb)
    A = rng.standard_normal((M, K)).astype(np.float32)
    B = rng.standard_normal((K, N)).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    resid = rng.standard_normal((M, N)).astype(np.float32)
    if dtype == 1:
        A, B = bf16_round(A), bf16_round(B)
    r8 = lambda n: (n + 7) // 8 * 8
    # storage: ta -> A kept as [K, M]; tb -> B kept as [K, N], else [N, K]; leading dims padded to 8
    As = pad_cols(A.T.copy(), r8(M)) if ta else pad_cols(A, r8(K))
    Bs = pad_cols(B, r8(N)) if tb else pad_cols(B.T.copy(), r8(K))
    tdt = torch.bfloat16 if dtype == 1 else torch.float32
    dA, dB = dev(As, tdt), dev(Bs, tdt)
    ldc = N + 3
    out = torch.zeros((M, ldc), dtype=torch.float32, device="cuda")
    out_act = torch.zeros((M, ldc), dtype=tdt, device="cuda")
    dres = dev(pad_cols(resid, ldc))
    H.hydra_op_gemm(dtype, ta, tb, M, N, K, 0.5, dA, As.shape[1], dB, Bs.shape[1], dev(bias), dres, out, out_act, ldc)
    torch.cuda.synchronize()
    ref = 0.5 * D.linear_fwd(A.astype(np.float64), B.astype(np.float64)) + bias + resid
    got = out.cpu().numpy()
    assert_close(got[:, :N], ref, 2e-5 if dtype == 0 else 1e-5, "gemm f32 out")
    assert (got[:, N:] == 0).all()                      # nothing written outside the result
    assert_close(out_act.float().cpu().numpy()[:, :N], ref, 1e-5 if dtype == 0 else 8e-3, "gemm act out")


@pytest.mark.parametrize("n", [1, 5, 1024, 1 << 20, (1 << 20) + 3])
def test_adam_kernel_against_oracle(H, n):
    rng = np.random.default_rng(n)
    w = rng.standard_normal(n).astype(np.float32) * 0.02
    m = rng.standard_normal(n).astype(np.float32) * 1e-3
    v = (rng.standard_normal(n).astype(np.float32) * 1e-3) ** 2
    g = rng.standard_normal(n).astype(np.float32) * 1e-2
    g[::7] = 0
    t, lr = 5, 3e-4
    dw, dm, dv, dg = dev(w), dev(m), dev(v), dev(g)
    shadow = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    H.hydra_op_adam(dw, dm, dv, dg, shadow, n, lr, 0.9, 0.999, 1e-8, t)
    torch.cuda.synchronize()
    rw, rm, rv = D.adam_update(w.astype(np.float64), m.astype(np.float64), v.astype(np.float64),
                               g.astype(np.float64), t, lr)
    assert_close(dm.cpu().numpy(), rm, 1e-6, "m")
    assert_close(dv.cpu().numpy(), rv, 1e-6, "v")
    assert_close(dw.cpu().numpy() - w, rw - w, 1e-4, "delta w")     # the update itself, not w
    assert (shadow.float().cpu().numpy() == bf16_round(dw.cpu().numpy())).all()
    # closed form: first step from zero state moves by -lr * g / (|g| + eps); zero gradient moves nothing
    z = torch.zeros(n, device="cuda")
    dw2, dm2, dv2 = dev(w), z.clone(), z.clone()
    H.hydra_op_adam(dw2, dm2, dv2, dg, None, n, lr, 0.9, 0.999, 1e-8, 1)
    torch.cuda.synchronize()
    w2 = dw2.cpu().numpy()
    assert (w2[g == 0] == w[g == 0]).all()
    nz = g != 0
    expect = -lr * g[nz].astype(np.float64) / (np.abs(g[nz].astype(np.float64)) + 1e-8)
    assert_close((w2 - w)[nz], expect, 2e-3 if n > 4 else 2e-2, "first step")


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("M,d", [(5, 8), (130, 136), (64, 768), (3, 4096)])
def test_layernorm_fwd(H, dtype, M, d):
    rng = np.random.default_rng(M + d)
    x = (rng.standard_normal((M, d)) * 2 + 0.5).astype(np.float32)
    g = (1 + 0.1 * rng.standard_normal(d)).astype(np.float32)
    b = (0.1 * rng.standard_normal(d)).astype(np.float32)
    tdt = torch.bfloat16 if dtype else torch.float32
    y = torch.zeros((M, d), dtype=tdt, device="cuda")
    mean = torch.zeros(M, device="cuda")
    rstd = torch.zeros(M, device="cuda")
    H.hydra_op_layernorm_fwd(dtype, dev(x), dev(g), dev(b), y, mean, rstd, M, d)
    torch.cuda.synchronize()
    ref, (xhat, rs) = D.layernorm_fwd(x.astype(np.float64), g.astype(np.float64), b.astype(np.float64))
    assert_close(y.float().cpu().numpy(), ref, 1e-5 if dtype == 0 else 8e-3, "ln out")
    assert_close(rstd.cpu().numpy(), rs[:, 0], 1e-5, "rstd")
    assert_close(mean.cpu().numpy(), x.astype(np.float64).mean(-1), 1e-5, "mean")


@pytest.mark.parametrize("with_res", [False, True])
@pytest.mark.parametrize("M,d", [(5, 8), (37, 200), (130, 768), (64, 1024), (19, 1600), (9, 2048)])
def test_layernorm_bwd_one_pass(H, M, d, with_res):
    """Backward of a LayerNorm in one pass: dx (with and without a residual gradient added), its bf16 copy, and the
    three column sums (dgamma, dbeta, sum of dx) against the oracle's formulas in float64; row counts that are not
    multiples of the kernel's row block, widths that fill 1 to 8 register chunks per lane."""
    rng = np.random.default_rng(1000 * M + d)
    x = (rng.standard_normal((M, d)) * 2 + 0.5).astype(np.float32)
    g = (1 + 0.1 * rng.standard_normal(d)).astype(np.float32)
    b = (0.1 * rng.standard_normal(d)).astype(np.float32)
    dy = rng.standard_normal((M, d)).astype(np.float32)
    res = rng.standard_normal((M, d)).astype(np.float32) if with_res else None
    y = torch.zeros((M, d), device="cuda")
    mean, rstd = torch.zeros(M, device="cuda"), torch.zeros(M, device="cuda")
    H.hydra_op_layernorm_fwd(0, dev(x), dev(g), dev(b), y, mean, rstd, M, d)
    dx = torch.full((M, d), float("nan"), device="cuda")
    dxh = torch.zeros((M, d), device="cuda", dtype=torch.bfloat16)
    dg, db, dc = (torch.full((d,), float("nan"), device="cuda") for _ in range(3))
    scratch = torch.empty(3 * d * ((M + 7) // 8), device="cuda")
    H.hydra_op_layernorm_bwd(dev(dy), dev(x), mean, rstd, dev(g), dev(res) if with_res else None, dx, dxh, dg, db, dc,
                             scratch, M, d)
    torch.cuda.synchronize()
    _, cache = D.layernorm_fwd(x.astype(np.float64), g.astype(np.float64), b.astype(np.float64))
    rdx, rdg, rdb = D.layernorm_bwd(dy.astype(np.float64), g.astype(np.float64), cache)
    if with_res:
        rdx = rdx + res.astype(np.float64)
    assert_close(dx.cpu().numpy(), rdx, 2e-5, "dx")
    assert_close(dxh.float().cpu().numpy(), rdx, 8e-3, "dx bf16")
    assert_close(dg.cpu().numpy(), rdg, 2e-5, "dgamma")
    assert_close(db.cpu().numpy(), rdb, 2e-5, "dbeta")
    assert_close(dc.cpu().numpy(), rdx.sum(axis=0), 2e-5, "column sum of dx")


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("n_mat,T", [(3, 8), (2, 72), (2, 264), (1, 520)])
def test_softmax_causal(H, dtype, n_mat, T):
    rng = np.random.default_rng(T)
    S = (rng.standard_normal((n_mat, T, T)) * 3).astype(np.float32)
    tdt = torch.bfloat16 if dtype else torch.float32
    P = torch.full((n_mat, T, T), 7.0, dtype=tdt, device="cuda")
    H.hydra_op_softmax_causal(dtype, dev(S), P, n_mat, T)
    torch.cuda.synchronize()
    got = P.float().cpu().numpy()
    mask = np.tril(np.ones((T, T), bool))
    s = np.where(mask, S.astype(np.float64), -np.inf)
    e = np.exp(s - s.max(-1, keepdims=True))
    ref = e / e.sum(-1, keepdims=True)
    i, j = np.nonzero(mask)
    assert_close(got[:, i, j], ref[:, i, j], 1e-5 if dtype == 0 else 8e-3, "softmax")
    # masked entries up to the end of the row's 256-wide diagonal block are exact zeros
    for r in range(T):
        zend = min(T, (r // 256 + 1) * 256)
        assert (got[:, r, r + 1:zend] == 0).all()
    if dtype == 0:
        assert np.abs(got[:, i, j].reshape(n_mat, -1).sum() - n_mat * T) < 1e-3 * n_mat * T


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("M,V", [(6, 32), (9, 1001), (4, 50257)])
def test_cross_entropy(H, dtype, M, V):
    rng = np.random.default_rng(V)
    logits = (rng.standard_normal((M, V)) * 2).astype(np.float32)
    tgt = rng.integers(0, V, M).astype(np.int32)
    tgt[1] = -1
    ld = (V + 63) // 64 * 64
    n = int((tgt >= 0).sum())
    tdt = torch.bfloat16 if dtype else torch.float32
    dl = torch.full((M, ld), 3.0, dtype=tdt, device="cuda")
    row = torch.zeros(M, device="cuda")
    H.hydra_op_cross_entropy(dtype, dev(pad_cols(logits, ld)), dev(tgt), row, dl, M, V, ld, 1.0 / n)
    torch.cuda.synchronize()
    loss, ref = D.cross_entropy(logits.astype(np.float64), tgt.reshape(1, M))
    got = dl.float().cpu().numpy()
    assert_close(got[:, :V], ref, 1e-5 if dtype == 0 else 8e-3, "dlogits")
    assert (got[:, V:] == 0).all() and (got[1] == 0).all()
    assert abs(float(row.cpu().numpy().astype(np.float64).sum()) / n - loss) < 1e-5 * max(1, abs(loss))
    # zero logits give ln V
    z = torch.zeros((M, ld), device="cuda")
    H.hydra_op_cross_entropy(0, z, dev(tgt), row, torch.zeros((M, ld), device="cuda"), M, V, ld, 1.0 / n)
    torch.cuda.synchronize()
    assert abs(float(row.cpu().numpy().sum()) / n - math.log(V)) < 1e-5


def test_single_slice_gemm_under_concurrency(H):
    """Contractions that fit one K slice (the head-width products of attention) skip the pipelined loop; their
    epilogue reuses the operand buffers in LDS and must wait for every wavefront of the block.  Two streams keep
    the device busy so that wavefronts of a block drift apart."""
    rng = np.random.default_rng(11)
    M, N, K = 512, 512, 64
    A = bf16_round(rng.standard_normal((M, K)).astype(np.float32))
    B = bf16_round(rng.standard_normal((N, K)).astype(np.float32))
    ref = A.astype(np.float64) @ B.astype(np.float64).T
    dA, dB = dev(A, torch.bfloat16), dev(B, torch.bfloat16)
    big = torch.randn((4096, 4096), device="cuda").to(torch.bfloat16)
    bigC = torch.empty((4096, 4096), device="cuda", dtype=torch.float32)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    outs = [torch.zeros((M, N), device="cuda", dtype=torch.float32) for _ in range(40)]
    torch.cuda.synchronize()
    for o in outs:
        H.hydra_op_gemm(1, 0, 0, 4096, 4096, 4096, 1.0, big, 4096, big, 4096, None, None, bigC, None, 4096, s2)
        H.hydra_op_gemm(1, 0, 0, M, N, K, 1.0, dA, K, dB, K, None, None, o, None, N, s1)
    torch.cuda.synchronize()
    for o in outs:
        assert_close(o.cpu().numpy(), ref, 1e-5, "single-slice gemm")


# products large enough for each tile shape the launcher picks for contraction-contiguous operands (256x256,
# 256x128 with eight wavefronts, 128x128, 128x64 in both pipeline depths), with and without ragged edges
LARGE_NT = [(1024, 12288, 1024), (1000, 12200, 512), (2048, 4096, 1024), (2000, 4100, 1024), (1024, 4096, 4096),
            (1000, 4000, 2048), (2048, 2304, 768), (2048, 768, 2304), (1100, 3000, 192),
            # a single, partly empty row of tiles: 256x128 (40 rows), 128x128 (100 rows), 256x256 (200 rows)
            (40, 26000, 128), (100, 30000, 2048), (200, 50000, 256),
            # and a single, partly empty column of tiles
            (52000, 120, 128), (30000, 100, 2048), (50000, 200, 256)]


@pytest.mark.parametrize("M,N,K", LARGE_NT)
def test_gemm_large_tiles_every_element(H, M, N, K):
    """Full-size products against the oracle's float64 product, every element of C: the fp32 and the bf16 output,
    scale, bias and residual included."""
    rng = np.random.default_rng(M + 3 * N + 7 * K)
    A = bf16_round(rng.standard_normal((M, K)).astype(np.float32))
    Bt = bf16_round(rng.standard_normal((N, K)).astype(np.float32))
    bias = rng.standard_normal(N).astype(np.float32)
    resid = rng.standard_normal((M, N)).astype(np.float32)
    out = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    out_act = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    H.hydra_op_gemm(1, 0, 0, M, N, K, 0.25, dev(A, torch.bfloat16), K, dev(Bt, torch.bfloat16), K, dev(bias),
                    dev(resid), out, out_act, N)
    torch.cuda.synchronize()
    ref = 0.25 * D.linear_fwd(A.astype(np.float64), Bt.T.astype(np.float64)) + bias + resid
    got = out.cpu().numpy().astype(np.float64)
    # element by element: fp32 accumulation of K products of magnitude ~1 and one rounding of the result
    tol = 4e-6 * np.sqrt(K) + 2e-7 * np.abs(ref)
    bad = np.abs(got - ref) > tol
    assert not bad.any(), f"{bad.sum()} elements of the fp32 result differ (worst {np.abs(got - ref).max():.3e})"
    got16 = out_act.float().cpu().numpy().astype(np.float64)
    bad = np.abs(got16 - ref) > tol + 2.0 ** -8 * np.abs(ref)          # one rounding to bf16 on top
    assert not bad.any(), f"{bad.sum()} elements of the bf16 result differ"


# weight-gradient shaped products (both operands stored with the contraction index strided, fp32 result, with and
# without accumulation into the result): several rounds of tiles, so that the tile groups an XCD walks wrap; ragged
# edges; the vocabulary-sized one of the LM head
LARGE_TN = [(4096, 8192, 1024), (1600, 6400, 1024), (1000, 3000, 520), (768, 50257, 2048), (16384, 1024, 256)]


@pytest.mark.parametrize("M,N,K", LARGE_TN)
def test_weight_gradient_products_every_element(H, M, N, K):
    rng = np.random.default_rng(5 * M + N + 11 * K)
    Kp, Np = (K + 7) // 8 * 8, (N + 7) // 8 * 8        # leading dimensions must be multiples of 8 elements
    A = bf16_round(rng.standard_normal((K, M)).astype(np.float32))      # x^T is wanted: A is stored [K, M]
    B = np.zeros((K, Np), np.float32)
    B[:, :N] = bf16_round(rng.standard_normal((K, N)).astype(np.float32))
    prev = rng.standard_normal((M, N)).astype(np.float32)
    ref = A.astype(np.float64).T @ B[:, :N].astype(np.float64)
    # Each fp32 addition into a running sum s_k of k unit-variance products rounds by up to 2^-24 |s_k| with |s_k| ~
    # sqrt(k), so the error of one element is a sum of K such terms: rms near 1e-8 K, with a heavy tail (plain
    # in-order fp32 summation on the CPU reaches 16 rms within 1e6 elements).  Tens of millions of elements are
    # compared here, hence 2.5e-7 K; a dropped or doubled product (magnitude ~1) is still 1000 times outside it.
    tol = 2.5e-7 * K
    for acc in (False, True):
        out = torch.from_numpy(prev.copy()).cuda()
        H.hydra_op_gemm(1, 1, 1, M, N, K, 1.0, dev(A, torch.bfloat16), M, dev(B, torch.bfloat16), Np, None,
                        out if acc else None, out, None, N)
        torch.cuda.synchronize()
        want = ref + prev if acc else ref
        got = out.cpu().numpy().astype(np.float64)
        bad = np.abs(got - want) > tol + 2e-7 * np.abs(want)
        assert not bad.any(), f"acc={acc}: {bad.sum()} elements differ (worst {np.abs(got - want).max():.3e})"


@pytest.mark.parametrize("M,N,K", [(2048, 4096, 1024), (1024, 4096, 4096), (2048, 2304, 768)])
def test_large_tile_gemms_repeat_bitwise_under_concurrency(H, M, N, K):
    """The tiles whose wavefront groups exchange partial sums through LDS (and the other direct-to-LDS tiles) while a
    second stream keeps the device busy: every repetition must give the same bits, and sampled rows the oracle's."""
    rng = np.random.default_rng(M + N + K)
    A = bf16_round(rng.standard_normal((M, K)).astype(np.float32))
    Bt = bf16_round(rng.standard_normal((N, K)).astype(np.float32))
    dA, dB = dev(A, torch.bfloat16), dev(Bt, torch.bfloat16)
    big = torch.randn((4096, 4096), device="cuda").to(torch.bfloat16)
    bigC = torch.empty((4096, 4096), device="cuda", dtype=torch.float32)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    outs = [torch.zeros((M, N), device="cuda", dtype=torch.float32) for _ in range(12)]
    torch.cuda.synchronize()
    for o in outs:
        H.hydra_op_gemm(1, 0, 0, 4096, 4096, 4096, 1.0, big, 4096, big, 4096, None, None, bigC, None, 4096, s2)
        H.hydra_op_gemm(1, 0, 0, M, N, K, 1.0, dA, K, dB, K, None, None, o, None, N, s1)
    torch.cuda.synchronize()
    for o in outs[1:]:
        assert torch.equal(o, outs[0])
    rows = np.array([0, 127, 128, 255, 256, M // 2 + 1, M - 1])
    ref = D.linear_fwd(A[rows].astype(np.float64), Bt.T.astype(np.float64))
    assert_close(outs[0][rows].cpu().numpy(), ref, 1e-5, "large gemm under concurrency")


@pytest.mark.parametrize("B,Hh,T,dh", [(2, 3, 72, 64), (1, 2, 264, 64), (2, 1, 136, 128), (1, 4, 512, 64), (1, 1, 8, 64)])
def test_fused_attention_forward_and_backward(H, B, Hh, T, dh):
    """Fused causal attention (scores, mask, softmax, PV in one kernel; backward without a stored probability
    matrix) against the oracle's attention on the same bf16-rounded operands: sequence lengths that are no
    multiple of the 64-key tile or the 128-row block, both head widths, several heads and samples."""
    rng = np.random.default_rng(B * 1000 + T + dh)
    d = Hh * dh
    M = B * T
    qkv = bf16_round(rng.standard_normal((M, 3 * d)).astype(np.float32))
    do = bf16_round(rng.standard_normal((M, d)).astype(np.float32) * 0.5)
    o_ref, cache = D.attention_fwd(qkv.astype(np.float64), B, T, Hh)
    q, k, v, p, scale = cache
    s = (q @ k.transpose(0, 1, 3, 2)) * scale
    s = np.where(np.tril(np.ones((T, T), dtype=bool)), s, -np.inf)
    smax = s.max(axis=-1)
    lse_ref = smax + np.log(np.exp(s - smax[..., None]).sum(axis=-1))          # [B,H,T]
    dqkv_ref = D.attention_bwd(do.astype(np.float64), cache, B, T, Hh)

    qkv_d = dev(qkv, torch.bfloat16)
    o_d = torch.full((M, d), float("nan"), device="cuda", dtype=torch.bfloat16)
    lse_d = torch.full((B * Hh * T,), float("nan"), device="cuda")
    H.hydra_op_attention_fwd(qkv_d, o_d, lse_d, B, Hh, T, dh)
    torch.cuda.synchronize()
    assert_close(o_d.float().cpu().numpy(), o_ref, 2e-2, "attention output")
    assert_close(lse_d.cpu().numpy().reshape(B, Hh, T), lse_ref, 1e-3, "log-sum-exp")

    do_d = dev(do, torch.bfloat16)
    dsum_d = torch.zeros(B * Hh * T, device="cuda")
    dqkv_d = torch.full((M, 3 * d), float("nan"), device="cuda", dtype=torch.bfloat16)
    H.hydra_op_attention_bwd(qkv_d, o_d, do_d, lse_d, dsum_d, dqkv_d, B, Hh, T, dh)
    torch.cuda.synchronize()
    got = dqkv_d.float().cpu().numpy()
    for name, sl in (("dq", slice(0, d)), ("dk", slice(d, 2 * d)), ("dv", slice(2 * d, 3 * d))):
        assert_close(got[:, sl], dqkv_ref[:, sl], 2e-2, name)
