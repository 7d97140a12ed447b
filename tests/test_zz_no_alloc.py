"""The LayerNorm backward entry point that allocates nothing (hmy_k_layernorm_bwd_static)
against the existing one with a caller's workspace (hmy_k_layernorm_bwd): same kernels, same
launch shape, so every output must be bit-identical; both are also held to the fp64 oracle.
Two calls in a row share the library's static workspace, the second on a smaller input."""
import numpy as np
import pytest
import torch

from oracle import model as om
from paper_2202_01306_amd import synth
from tests.helpers import max_rel_err

pytestmark = pytest.mark.gpu

PRECS = [("fp32", 0, torch.float32, 1e-4), ("bf16", 1, torch.bfloat16, 2e-2)]


def _case(B, prec, pc, dt, tol, T, d, seed):
    print(f"layernorm_bwd_static {prec} T={T} d={d}", flush=True)
    rng = np.random.default_rng(seed)

    def rnd(shape, scale=1.0):
        a = (rng.standard_normal(shape) * scale).astype(np.float32)
        return synth.round_bf16(a) if prec == "bf16" else a

    def dev(a, dtype):
        return torch.from_numpy(np.ascontiguousarray(a)).to(device="cuda", dtype=dtype)

    def host(t):
        torch.cuda.synchronize()
        return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)

    # x, res and dx are the fp32 residual stream; dy, gamma, beta have the element type
    x, g, bt = (rng.standard_normal((T, d)) * 2.0).astype(np.float32), rnd((d,)) + 1, rnd((d,), 0.1)
    g = synth.round_bf16(g) if prec == "bf16" else g
    dy, res = rnd((T, d)), rng.standard_normal((T, d)).astype(np.float32)
    dg0, db0 = rng.standard_normal(d).astype(np.float32), rng.standard_normal(d).astype(np.float32)
    xd, gd, bd, dyd, resd = dev(x, torch.float32), dev(g, dt), dev(bt, dt), dev(dy, dt), dev(res, torch.float32)
    y = torch.empty(T, d, device="cuda", dtype=dt)
    mean, rstd = torch.empty(T, device="cuda"), torch.empty(T, device="cuda")
    B.hmy_k_layernorm_fwd(pc, xd, gd, bd, y, mean, rstd, T, d, synth.LN_EPS)
    # the existing entry point, with a workspace of the caller's
    ws = torch.full((256 * 2 * d,), float("nan"), device="cuda")
    dx_a, dg_a, db_a = torch.empty_like(xd), dev(dg0, torch.float32), dev(db0, torch.float32)
    B.hmy_k_layernorm_bwd(pc, dyd, xd, mean, rstd, gd, resd, dx_a, dg_a, db_a, T, d, workspace=ws)
    # the entry point that allocates nothing
    dx_b, dg_b, db_b = torch.empty_like(xd), dev(dg0, torch.float32), dev(db0, torch.float32)
    B.hmy_k_layernorm_bwd_static(pc, dyd, xd, mean, rstd, gd, resd, dx_b, dg_b, db_b, T, d)
    torch.cuda.synchronize()
    assert torch.equal(dx_a, dx_b) and torch.equal(dg_a, dg_b) and torch.equal(db_a, db_b)
    _, (xhat, rs) = om.layernorm_fwd(x.astype(np.float64), g.astype(np.float64), bt.astype(np.float64), synth.LN_EPS)
    dxr, dgr, dbr = om.layernorm_bwd(dy.astype(np.float64), (xhat, rs), g.astype(np.float64))
    etol = tol if prec == "bf16" else 2e-5
    assert max_rel_err(host(dx_b), dxr + res) < (tol if prec == "bf16" else 2e-5)
    assert max_rel_err(host(dg_b) - dg0, dgr) < etol
    assert max_rel_err(host(db_b) - db0, dbr) < etol


@pytest.mark.parametrize("prec,pc,dt,tol", PRECS)
def test_static_workspace_matches_the_callers_workspace_on_two_calls_in_a_row(prec, pc, dt, tol):
    from paper_2202_01306_amd import binding as B
    _case(B, prec, pc, dt, tol, 3000, 1024, 1)   # 256 workgroups: every row of the static workspace is used
    _case(B, prec, pc, dt, tol, 37, 256, 2)      # smaller: fewer, shorter rows over the first call's leftovers
    _case(B, prec, pc, dt, tol, 130, 4096 if prec == "bf16" else 2048, 3)   # wide rows: several waves share a row


def test_static_workspace_rejects_rows_beyond_its_limit():
    from paper_2202_01306_amd import binding as B
    T, d = 4, 4104
    z = torch.zeros(T, d, device="cuda")
    v = torch.zeros(d, device="cuda")
    r = torch.zeros(T, device="cuda")
    with pytest.raises(B.HmyError) as e:
        B.hmy_k_layernorm_bwd_static(0, z, z, r, r, v, None, z, v, v, T, d)
    assert "4096" in str(e.value)
