"""The entry point that allocates nothing (hydra_op_layernorm_bwd_static: partial sums in a fixed device array
instead of a caller-supplied workspace) against the entry point it is a variant of, through the C ABI: two calls in
a row, the second on a smaller input, each bit for bit equal to hydra_op_layernorm_bwd on the same input and within
tolerance of the oracle's float64 formulas; sizes beyond the array are refused."""
import numpy as np
import pytest

from oracle import decoder as D
from tests.parity_utils import assert_close

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _case(H, M, d, seed, with_res, static):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((M, d)) * 2 + 0.5).astype(np.float32)
    g = (1 + 0.1 * rng.standard_normal(d)).astype(np.float32)
    b = (0.1 * rng.standard_normal(d)).astype(np.float32)
    dy = rng.standard_normal((M, d)).astype(np.float32)
    res = rng.standard_normal((M, d)).astype(np.float32) if with_res else None
    dev = lambda a: torch.from_numpy(a).cuda()
    xd, gd, dyd = dev(x), dev(g), dev(dy)
    rd = dev(res) if with_res else None
    y = torch.zeros((M, d), device="cuda")
    mean, rstd = torch.zeros(M, device="cuda"), torch.zeros(M, device="cuda")
    H.hydra_op_layernorm_fwd(0, xd, gd, dev(b), y, mean, rstd, M, d)
    dx = torch.full((M, d), float("nan"), device="cuda")
    dxh = torch.zeros((M, d), device="cuda", dtype=torch.bfloat16)
    dg, db, dc = (torch.full((d,), float("nan"), device="cuda") for _ in range(3))
    if static:
        torch.cuda.synchronize()
        # torch's count of allocations made so far (it only grows; bytes in use may fall when the collector frees
        # garbage of earlier tests at this very moment)
        before = torch.cuda.memory_stats()["allocation.all.allocated"]
        H.hydra_op_layernorm_bwd_static(dyd, xd, mean, rstd, gd, rd, dx, dxh, dg, db, dc, M, d)
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
    else:
        scratch = torch.empty(3 * d * ((M + 7) // 8), device="cuda")
        H.hydra_op_layernorm_bwd(dyd, xd, mean, rstd, gd, rd, dx, dxh, dg, db, dc, scratch, M, d)
    torch.cuda.synchronize()
    out = [t.cpu().numpy() for t in (dx, dg, db, dc)] + [dxh.float().cpu().numpy()]
    _, cache = D.layernorm_fwd(x.astype(np.float64), g.astype(np.float64), b.astype(np.float64))
    rdx, rdg, rdb = D.layernorm_bwd(dy.astype(np.float64), g.astype(np.float64), cache)
    if with_res:
        rdx = rdx + res.astype(np.float64)
    return out, (rdx, rdg, rdb, rdx.sum(axis=0))


def test_static_scratch_entry_point_equals_the_workspace_one():
    from paper_2110_08633_amd import hydra as H
    # two calls in a row on the same GPU, the second smaller (fewer row blocks and narrower rows than the first
    # left in the array), then a third, larger again
    for M, d, seed, with_res in ((1027, 768, 1, True), (37, 200, 2, False), (2048, 1024, 3, True)):
        got, ref = _case(H, M, d, seed, with_res, static=True)
        want, _ = _case(H, M, d, seed, with_res, static=False)
        for a, b, name in zip(got, want, ("dx", "dgamma", "dbeta", "colsum dx", "dx bf16")):
            assert np.isfinite(a).all() and (a == b).all(), (M, d, name)
        for a, r, name in zip(got[:4], ref, ("dx", "dgamma", "dbeta", "colsum dx")):
            assert_close(a, r, 2e-5, f"{M}x{d} {name}")
        assert_close(got[4], ref[0], 8e-3, f"{M}x{d} dx bf16")


def test_static_scratch_entry_point_refuses_sizes_beyond_its_array():
    from paper_2110_08633_amd import hydra as H
    M, d = 8 * 400, 2048            # 3 * 2048 * 400 = 2 457 600 floats > 2 Mi
    z = torch.zeros((M, d), device="cuda")
    v = torch.zeros(M, device="cuda")
    c = torch.zeros(d, device="cuda")
    with pytest.raises(H.HydraError) as e:
        H.hydra_op_layernorm_bwd_static(z, z, v, v, c, None, z, None, c, c, None, M, d)
    assert e.value.code == H.E_INVAL
    with pytest.raises(H.HydraError) as e:
        H.hydra_op_layernorm_bwd_static(z, z, v, v, c, None, z, None, c, c, None, 64, 2052)   # row wider than supported
    assert e.value.code == H.E_INVAL
