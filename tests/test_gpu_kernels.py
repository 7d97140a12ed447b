"""GPU parity of every single-kernel entry point of the C ABI against the fp64
oracle, element by element, on seeded inputs spanning several tiles and ragged
tails.  Metric: max|x - ref| / max|ref| per tensor.  Tolerances: fp32 path 1e-4
(2e-5 for pure elementwise ops); bf16 path 2e-2."""
import math

import numpy as np
import pytest
import torch

from oracle import model as om
from paper_2202_01306_amd import synth
from tests.helpers import max_rel_err

pytestmark = pytest.mark.gpu

B = None


@pytest.fixture(scope="module", autouse=True)
def _binding():
    global B
    from paper_2202_01306_amd import binding
    B = binding
    yield
    torch.cuda.synchronize()


PRECS = [("fp32", 0, torch.float32, 1e-4), ("bf16", 1, torch.bfloat16, 2e-2)]


def rnd(rng, shape, prec, scale=1.0):
    """Random fp32 values, rounded to bf16 first in bf16 mode so both sides start equal."""
    a = (rng.standard_normal(shape) * scale).astype(np.float32)
    return synth.round_bf16(a) if prec == "bf16" else a


def dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a)).to(device="cuda", dtype=dtype)


def host(t):
    torch.cuda.synchronize()
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("prec,pc,dt,tol", PRECS)
@pytest.mark.parametrize("T,d", [(5, 128), (130, 1024), (67, 1600), (33, 4096), (1037, 1600), (70, 2056), (9, 8192)])
def test_layernorm_fwd_bwd(prec, pc, dt, tol, T, d):
    say(f"layernorm {prec} T={T} d={d}")
    rng = np.random.default_rng(T * 1000 + d)
    # the residual stream (x, res, dx) is fp32 in every precision; dy, gamma, beta and y have the element type
    x = (rng.standard_normal((T, d)) * 2.0 + 0.5).astype(np.float32)
    g, bt = rnd(rng, (d,), prec) + 1, rnd(rng, (d,), prec, 0.1)
    g = synth.round_bf16(g) if prec == "bf16" else g
    dy, res = rnd(rng, (T, d), prec), rng.standard_normal((T, d)).astype(np.float32)
    xd, gd, bd = dev(x, torch.float32), dev(g, dt), dev(bt, dt)
    y = torch.empty(T, d, device="cuda", dtype=dt)
    mean = torch.empty(T, device="cuda")
    rstd = torch.empty(T, device="cuda")
    B.hmy_k_layernorm_fwd(pc, xd, gd, bd, y, mean, rstd, T, d, synth.LN_EPS)
    yr, (xhat, rs) = om.layernorm_fwd(x.astype(np.float64), g.astype(np.float64), bt.astype(np.float64), synth.LN_EPS)
    assert max_rel_err(host(y), yr) < (tol if prec == "bf16" else 2e-5)
    assert max_rel_err(host(mean), x.astype(np.float64).mean(axis=1)) < 1e-5
    assert max_rel_err(host(rstd), rs[:, 0]) < 1e-5
    # backward, accumulating onto non-zero dgamma / dbeta, residual added, in place over res
    dg0, db0 = rng.standard_normal(d).astype(np.float32), rng.standard_normal(d).astype(np.float32)
    dgd, dbd = dev(dg0, torch.float32), dev(db0, torch.float32)
    resd = dev(res, torch.float32)
    low = torch.zeros(T, d, device="cuda", dtype=dt)
    B.hmy_k_layernorm_bwd(pc, dev(dy, dt), xd, mean, rstd, gd, resd, resd, dgd, dbd, T, d, dx_e=low)
    dxr, dgr, dbr = om.layernorm_bwd(dy.astype(np.float64), (xhat, rs), g.astype(np.float64))
    assert max_rel_err(host(resd), dxr + res) < (tol if prec == "bf16" else 2e-5)
    assert torch.equal(low, resd.to(dt))        # the element-typed copy is the rounding of what was stored
    assert max_rel_err(host(dgd) - dg0, dgr) < (tol if prec == "bf16" else 2e-5)
    assert max_rel_err(host(dbd) - db0, dbr) < (tol if prec == "bf16" else 2e-5)
    # without residual
    dxd = torch.empty_like(xd)
    B.hmy_k_layernorm_bwd(pc, dev(dy, dt), xd, mean, rstd, gd, None, dxd, dgd, dbd, T, d)
    assert max_rel_err(host(dxd), dxr) < tol
    # with a workspace: partial sums per workgroup, added up by a second kernel
    dgd2, dbd2 = dev(dg0, torch.float32), dev(db0, torch.float32)
    ws = torch.full((256 * 2 * d,), float("nan"), device="cuda")
    B.hmy_k_layernorm_bwd(pc, dev(dy, dt), xd, mean, rstd, gd, None, dxd, dgd2, dbd2, T, d, workspace=ws)
    assert max_rel_err(host(dxd), dxr) < tol
    assert max_rel_err(host(dgd2) - dg0, dgr) < (tol if prec == "bf16" else 2e-5)
    assert max_rel_err(host(dbd2) - db0, dbr) < (tol if prec == "bf16" else 2e-5)
    # the column sums of the residual gradient taken along (a bias gradient), in place over res, with and
    # without the workspace; everything else as before
    for ws in (None, torch.full((256 * 3 * d,), float("nan"), device="cuda")):
        dgd3, dbd3 = dev(dg0, torch.float32), dev(db0, torch.float32)
        s0 = rng.standard_normal(d).astype(np.float32)
        sd, resd = dev(s0, torch.float32), dev(res, torch.float32)
        B.hmy_k_layernorm_bwd(pc, dev(dy, dt), xd, mean, rstd, gd, resd, resd, dgd3, dbd3, T, d, workspace=ws, dres_sum=sd)
        assert max_rel_err(host(sd) - s0, res.astype(np.float64).sum(axis=0)) < 1e-5
        assert max_rel_err(host(resd), dxr + res) < (tol if prec == "bf16" else 2e-5)
        assert max_rel_err(host(dgd3) - dg0, dgr) < (tol if prec == "bf16" else 2e-5)
        assert max_rel_err(host(dbd3) - db0, dbr) < (tol if prec == "bf16" else 2e-5)
    with pytest.raises(B.HmyError):      # sums of a residual that is not there
        B.hmy_k_layernorm_bwd(pc, dev(dy, dt), xd, mean, rstd, gd, None, dxd, dgd, dbd, T, d, dres_sum=dgd2)


@pytest.mark.parametrize("prec,pc,dt,tol", PRECS)
def test_gelu_fwd_bwd(prec, pc, dt, tol):
    say(f"gelu {prec}")
    rng = np.random.default_rng(1)
    n = 8 * 12345
    u, dg = rnd(rng, (n,), prec, 2.5), rnd(rng, (n,), prec)
    ud = dev(u, dt)
    g = torch.empty_like(ud)
    B.hmy_k_gelu_fwd(pc, ud, g, n)
    assert max_rel_err(host(g), om.gelu_fwd(u.astype(np.float64))) < (tol if prec == "bf16" else 2e-6)
    dgd = dev(dg, dt)
    B.hmy_k_gelu_bwd(pc, dgd, ud, dgd, n)     # in place
    assert max_rel_err(host(dgd), om.gelu_bwd(dg.astype(np.float64), u.astype(np.float64))) < (tol if prec == "bf16" else 2e-6)


@pytest.mark.parametrize("prec,pc,dt,tol", PRECS)
@pytest.mark.parametrize("T,N", [(3, 8), (257, 3072), (1000, 136), (4096, 4096)])
def test_gelu_bwd_with_column_sums(prec, pc, dt, tol, T, N):
    say(f"gelu backward + column sums {prec} {T}x{N}")
    rng = np.random.default_rng(T * 3 + N)
    u, dg = rnd(rng, (T, N), prec, 2.5), rnd(rng, (T, N), prec)
    db0 = rng.standard_normal(N).astype(np.float32)
    ud, dgd, dbd = dev(u, dt), dev(dg, dt), dev(db0, torch.float32)
    B.hmy_k_gelu_bwd_colsum(pc, dgd, ud, dgd, dbd, T, N)     # in place, as the engine runs it
    ref = om.gelu_bwd(dg.astype(np.float64), u.astype(np.float64))
    assert max_rel_err(host(dgd), ref) < (tol if prec == "bf16" else 2e-6)
    # the sums are those of the stored values, exactly what a separate pass over du would have added
    assert max_rel_err(host(dbd) - db0, host(dgd).astype(np.float64).sum(axis=0)) < 1e-5
    same = dev(dg, dt)
    B.hmy_k_gelu_bwd(pc, same, ud, same, T * N)
    assert torch.equal(same, dgd)


@pytest.mark.parametrize("prec,pc,dt,tol", PRECS)
@pytest.mark.parametrize("T,N", [(3, 8), (257, 3072), (1000, 136)])
def test_colsum_accumulates(prec, pc, dt, tol, T, N):
    say(f"colsum {prec} {T}x{N}")
    rng = np.random.default_rng(T + N)
    a = rnd(rng, (T, N), prec)
    out0 = rng.standard_normal(N).astype(np.float32)
    out = dev(out0, torch.float32)
    B.hmy_k_colsum(pc, dev(a, dt), out, T, N)
    assert max_rel_err(host(out) - out0, a.astype(np.float64).sum(axis=0)) < 1e-5


@pytest.mark.parametrize("prec,pc,dt,tol", PRECS)
def test_embedding_fwd_bwd_with_repeated_ids(prec, pc, dt, tol):
    say(f"embed {prec}")
    rng = np.random.default_rng(2)
    b, s, d, V = 3, 40, 64, 50
    T = b * s
    ids = rng.integers(0, V, size=(b, s), dtype=np.int32)       # 120 draws from 50 ids: many repeats
    wte, wpe = rnd(rng, (V, d), prec), rnd(rng, (s, d), prec)
    x = torch.empty(T, d, device="cuda", dtype=torch.float32)     # the residual stream starts here: fp32
    idd = torch.from_numpy(ids.reshape(-1)).cuda()
    B.hmy_k_embed_fwd(pc, idd, dev(wte, dt), dev(wpe, dt), x, T, d, s, V)
    params = {"wte": wte.astype(np.float64), "wpe": wpe.astype(np.float64)}
    spec = om.Spec(1, d, 1, 8, s, V)
    xr, cache = om.embed_fwd(ids, params, spec)
    assert max_rel_err(host(x), xr) < 1e-6         # a sum of two exactly representable values
    dx = rng.standard_normal((T, d)).astype(np.float32)
    dwte = torch.zeros(V, d, device="cuda")
    dwpe = torch.zeros(s, d, device="cuda")
    B.hmy_k_embed_bwd(pc, idd, dev(dx, torch.float32), dwte, dwpe, T, d, s, V)
    _, g = om.embed_bwd(dx.astype(np.float64), cache, params, spec)
    assert max_rel_err(host(dwte), g["wte"]) < 1e-5
    assert max_rel_err(host(dwpe), g["wpe"]) < 1e-5


def _gemm_case(prec, pc, dt, tol, M, N, K, ta, tb, c_fp32, accumulate, bias, res, gelu, use_mfma, pad=0, res_fp32=0,
               row_pad=0, ldc=None):
    rng = np.random.default_rng(M * 7 + N * 3 + K + ta * 2 + tb)
    lda = M + row_pad if ta else K + pad        # pad: rows whose contiguous axis is K; row_pad: A stored [K, M]
    ldb = N if tb else K + pad
    A = rnd(rng, (K, lda) if ta else (M, lda), prec)
    Bm = rnd(rng, (K, ldb) if tb else (N, ldb), prec)
    A64 = (A[:, :M].T if ta else A[:, :K]).astype(np.float64)         # [M,K]
    B64 = (Bm[:, :N] if tb else Bm[:, :K].T).astype(np.float64)       # [K,N]
    ref = A64 @ B64
    biasv = rnd(rng, (N,), prec) if bias else None
    resv = (rng.standard_normal((M, N)).astype(np.float32) if res_fp32 else rnd(rng, (M, N), prec)) if res else None
    if bias:
        ref = ref + biasv
    if res:
        ref = ref + resv
    ldc = ldc or N + (8 if pad else 0)
    cdt = torch.float32 if c_fp32 else dt
    c0 = rng.standard_normal((M, ldc)).astype(np.float32)
    Cd = dev(c0, cdt)
    if accumulate:
        ref = ref + host(Cd)[:, :N]
    gout = torch.zeros(M, ldc, device="cuda", dtype=dt) if gelu else None
    if gelu == "in place":
        gout = Cd                       # only gelu(C) is wanted: it replaces C
    B.hmy_set_kernel_path(use_mfma)
    try:
        B.hmy_k_gemm(pc, M, N, K, dev(A, dt), lda, dev(Bm, dt), ldb, Cd, ldc, ta=ta, tb=tb, c_fp32=c_fp32,
                     accumulate=accumulate, bias=dev(biasv, dt) if bias else None,
                     res=dev(resv, torch.float32 if res_fp32 else dt) if res else None, ldr=N, gelu_out=gout,
                     res_fp32=res_fp32)
        got = host(Cd)
    finally:
        B.hmy_set_kernel_path(True)
    scale = math.sqrt(K)   # entries are sums of K unit-variance products
    if gelu == "in place":
        gref = om.gelu_fwd(synth.round_bf16(ref.astype(np.float32)).astype(np.float64) if prec == "bf16" else ref)
        # where the rounding of C falls on the other side the activation moves by one bf16 step of C
        assert np.abs(got[:, :N] - gref).max() / max(np.abs(gref).max(), scale) < tol, "gelu in place"
        return
    assert np.abs(got[:, :N] - ref).max() / max(np.abs(ref).max(), scale) < tol, "C"
    if ldc > N:   # columns beyond N are never written
        assert np.array_equal(got[:, N:], host(dev(c0, cdt))[:, N:])
    if gelu:
        gref = om.gelu_fwd(got[:, :N])          # gelu of the stored (rounded) C
        assert max_rel_err(host(gout)[:, :N], gref) < tol


GEMM_SHAPES = [(200, 136, 72), (128, 128, 32), (130, 257, 1001), (136, 264, 1001), (1, 8, 8), (384, 128, 512)]


@pytest.mark.parametrize("use_mfma", [True, False])
@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 1), (1, 0)])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_bf16_all_layouts(use_mfma, ta, tb, M, N, K):
    say(f"gemm bf16 mfma={use_mfma} ta={ta} tb={tb} {M}x{N}x{K}")
    pad = 7 if K == 1001 else 0     # makes every leading dimension a multiple of 8
    ragged_rows = (ta and M % 8) or (tb and N % 8)     # an operand stored [K, rows] whose rows are not 16-byte multiples
    if ragged_rows and use_mfma:
        # the matrix-core kernels cannot take it, and the library says so instead of quietly running the plain kernel
        with pytest.raises(B.HmyError) as e:
            _gemm_case("bf16", 1, torch.bfloat16, 2e-2, M, N, K, ta, tb, 0, 0, False, False, False, use_mfma, pad)
        assert e.value.code == B.HMY_E_INVALID and "16-byte aligned" in str(e.value)
        return
    _gemm_case("bf16", 1, torch.bfloat16, 2e-2, M, N, K, ta, tb, 0, 0, False, False, False, use_mfma, pad)


@pytest.mark.parametrize("use_mfma", [True, False])
def test_gemm_bf16_epilogues(use_mfma):
    say(f"gemm bf16 epilogues mfma={use_mfma}")
    args = ("bf16", 1, torch.bfloat16, 2e-2)
    _gemm_case(*args, 200, 136, 72, 0, 0, 0, 0, True, False, False, use_mfma)       # bias
    _gemm_case(*args, 200, 136, 72, 0, 0, 0, 0, True, True, False, use_mfma)        # bias + residual
    _gemm_case(*args, 200, 136, 72, 0, 0, 1, 0, True, True, False, use_mfma, res_fp32=1)    # ... on the fp32 residual stream
    _gemm_case(*args, 384, 256, 128, 0, 0, 1, 0, True, True, False, use_mfma, res_fp32=1)   # ... whole tiles (16-byte accesses)
    _gemm_case(*args, 256, 128, 1024, 0, 0, 1, 0, True, True, False, use_mfma, res_fp32=1)  # ... one tile per workgroup, K tile 64
    _gemm_case(*args, 200, 136, 72, 0, 0, 0, 0, True, False, True, use_mfma)        # bias + gelu output
    _gemm_case(*args, 200, 136, 72, 0, 0, 0, 0, True, False, "in place", use_mfma)  # bias + gelu, the only output
    _gemm_case(*args, 384, 256, 128, 0, 0, 0, 0, True, False, "in place", use_mfma) # ... on whole tiles (16-byte stores)
    _gemm_case(*args, 200, 136, 72, 0, 0, 1, 0, False, False, False, use_mfma)      # fp32 C (logits)
    _gemm_case(*args, 136, 72, 200, 1, 1, 1, 1, False, False, False, use_mfma)      # wgrad: fp32 C +=
    _gemm_case(*args, 100, 1001, 64, 0, 0, 1, 0, False, False, False, use_mfma, 8)  # ragged N, padded ldc and lda
    _gemm_case(*args, 1000, 64, 96, 1, 1, 1, 1, False, False, False, use_mfma)      # ragged M (vocab-like), K=96


@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 1), (1, 0)])
@pytest.mark.parametrize("K", [96, 320])
def test_gemm_bf16_large_outputs_all_layouts(ta, tb, K):
    """Outputs large enough for the 256x256 block tile (one workgroup per compute unit or more), with a ragged last
    tile row and column; K of fewer and of more tiles than the ring has stages."""
    say(f"gemm bf16 large ta={ta} tb={tb} K={K}")
    _gemm_case("bf16", 1, torch.bfloat16, 2e-2, 3600, 3336, K, ta, tb, 0, 0, False, False, False, True)


def test_gemm_bf16_large_outputs_epilogues():
    args = ("bf16", 1, torch.bfloat16, 2e-2)
    say("gemm bf16 large: bias + gelu")
    _gemm_case(*args, 4096, 3072, 64, 0, 0, 0, 0, True, False, True, True)
    say("gemm bf16 large: bias + gelu in place")
    _gemm_case(*args, 4096, 3072, 64, 0, 0, 0, 0, True, False, "in place", True)
    say("gemm bf16 large: bias + fp32 residual stream")
    _gemm_case(*args, 4096, 3072, 160, 0, 0, 1, 0, True, True, False, True, res_fp32=1)
    say("gemm bf16 large: bias + bf16 residual")
    _gemm_case(*args, 4096, 3072, 64, 0, 0, 0, 0, True, True, False, True)
    say("gemm bf16 large: fp32 C +=")
    _gemm_case(*args, 3072, 4096, 128, 1, 1, 1, 1, False, False, False, True)
    _gemm_case(*args, 50257, 1024, 96, 1, 1, 1, 1, False, False, False, True, row_pad=47)   # vocabulary rows, ragged
    say("gemm bf16: fp32 C +=, contraction split over workgroups (128x128 tiles)")
    _gemm_case(*args, 1024, 1024, 4096, 1, 1, 1, 1, False, False, False, True)
    _gemm_case(*args, 1536, 1024, 2048 + 32, 0, 1, 1, 1, False, False, False, True)    # the last split has two K tiles
    say("gemm bf16 large: fp32 logits, ragged vocabulary, padded leading dimensions")
    _gemm_case(*args, 512, 50257, 64, 0, 0, 1, 0, False, False, False, True, 8)


def test_gemm_bf16_tiles_that_stick_out_of_c():
    """Outputs whose width is no multiple of the block tile, with 16-byte aligned rows: whole groups of 8 columns of an
    edge tile leave through the vector path, a ragged last group element by element; nothing beyond N is written."""
    args = ("bf16", 1, torch.bfloat16, 2e-2)
    say("gemm bf16 edge tiles: fp32 C, ragged width, aligned rows")
    _gemm_case(*args, 200, 333, 128, 0, 0, 1, 0, False, False, False, True, ldc=336)
    _gemm_case(*args, 200, 333, 128, 0, 0, 1, 1, False, False, False, True, ldc=336)      # +=
    say("gemm bf16 edge tiles: bf16 C, bias + gelu, ragged width")
    _gemm_case(*args, 200, 333, 128, 0, 0, 0, 0, True, False, True, True, ldc=336)
    say("gemm bf16 edge tiles: 1600 wide, bias + fp32 residual stream")
    _gemm_case(*args, 2048, 1600, 64, 0, 0, 1, 0, True, True, False, True, res_fp32=1)
    _gemm_case(*args, 1600, 1608, 256, 1, 1, 1, 1, False, False, False, True)            # weight gradient, ragged rows too
    say("gemm bf16 edge tiles, 256x256: fp32 C with a ragged width; bf16 C with bias + gelu")
    _gemm_case(*args, 4096, 2999, 64, 0, 0, 1, 0, False, False, False, True, ldc=3008)
    _gemm_case(*args, 4000, 3000, 96, 0, 0, 0, 0, True, False, True, True)
    _gemm_case(*args, 4000, 3000, 64, 0, 1, 0, 0, True, True, False, True)


@pytest.mark.parametrize("ta,tb", [(0, 0), (0, 1), (1, 1)])
def test_gemm_fp32(ta, tb):
    say(f"gemm fp32 ta={ta} tb={tb}")
    args = ("fp32", 0, torch.float32, 1e-5)
    _gemm_case(*args, 130, 72, 100, ta, tb, 0, 0, True, True, False, True)
    _gemm_case(*args, 64, 200, 33, ta, tb, 1, 1, False, False, False, True)
    _gemm_case(*args, 128, 512, 128, ta, tb, 0, 0, True, False, True, True)
    _gemm_case(*args, 128, 512, 128, ta, tb, 0, 0, True, False, "in place", True)


def test_gemm_rejects_bad_arguments():
    a = torch.zeros(64, 64, device="cuda", dtype=torch.bfloat16)
    with pytest.raises(B.HmyError) as e:
        B.hmy_k_gemm(1, 64, 64, 64, a, 32, a, 64, a, 64)       # lda < K
    assert e.value.code == B.HMY_E_INVALID
    with pytest.raises(B.HmyError):
        B.hmy_k_gemm(1, 64, 64, 64, a, 64, a, 64, a, 64, accumulate=1)   # accumulate needs fp32 C
    with pytest.raises(B.HmyError):
        B.hmy_k_gemm(1, 0, 64, 64, a, 64, a, 64, a, 64)


@pytest.mark.parametrize("prec,pc,dt,tol,use_mfma", [p + (True,) for p in PRECS] + [PRECS[1] + (False,)])
@pytest.mark.parametrize("causal", [1, 0])
@pytest.mark.parametrize("b,s,H,dh", [(2, 64, 2, 32), (1, 100, 3, 64), (2, 256, 1, 128), (1, 7, 2, 64),
                                      (1, 333, 2, 64), (2, 130, 2, 32), (1, 161, 1, 128)])
def test_attention_fwd_bwd(prec, pc, dt, tol, use_mfma, causal, b, s, H, dh):
    say(f"attention {prec} mfma={use_mfma} causal={causal} b={b} s={s} H={H} dh={dh}")
    B.hmy_set_kernel_path(use_mfma)
    try:
        _attention_case(prec, pc, dt, tol, causal, b, s, H, dh)
    finally:
        B.hmy_set_kernel_path(True)


def _attention_case(prec, pc, dt, tol, causal, b, s, H, dh):
    rng = np.random.default_rng(s * 10 + dh + causal)
    d = H * dh
    T = b * s
    qkv = rnd(rng, (T, 3 * d), prec, 1.5)
    spec = om.Spec(1, d, H, 8, s, 16, bool(causal))
    oref, cache = om.attention_fwd(qkv.astype(np.float64), spec, b)
    qd = dev(qkv, dt)
    o = torch.empty(T, d, device="cuda", dtype=dt)
    lse = torch.empty(b * H * s, device="cuda")
    B.hmy_k_attn_fwd(pc, qd, o, lse, b, s, H, dh, causal)
    assert max_rel_err(host(o), oref) < tol
    # logsumexp of the scaled, masked scores
    q, k, v, P = cache
    S = (q @ k.transpose(0, 1, 3, 2)) / math.sqrt(dh)
    if causal:
        S = np.where(np.triu(np.ones((s, s), bool), 1), -np.inf, S)
    mx = S.max(-1)
    lref = mx + np.log(np.exp(S - mx[..., None]).sum(-1))
    assert np.abs(host(lse).reshape(b, H, s) - lref).max() < (3e-2 if prec == "bf16" else 1e-4)
    # backward consumes the kernel's own o and lse (as the executor does)
    do = rnd(rng, (T, d), prec)
    dqkv = torch.full((T, 3 * d), float("nan"), device="cuda", dtype=dt)
    delta = torch.empty(b * H * s, device="cuda")
    B.hmy_k_attn_bwd(pc, qd, o, dev(do, dt), lse, delta, dqkv, b, s, H, dh, causal)
    ref = om.attention_bwd(do.astype(np.float64), cache, spec, b)
    got = host(dqkv)
    for name, sl in (("dq", slice(0, d)), ("dk", slice(d, 2 * d)), ("dv", slice(2 * d, 3 * d))):
        assert max_rel_err(got[:, sl], ref[:, sl]) < tol, name
    # once more with the bias gradient of the QKV projection taken along: the column sums of dqkv as stored, added
    # onto what is there; dqkv and delta as before
    db0 = rng.standard_normal(3 * d).astype(np.float32)
    dbd = dev(db0, torch.float32)
    dqkv2 = torch.full((T, 3 * d), float("nan"), device="cuda", dtype=dt)
    delta2 = torch.full((b * H * s,), float("nan"), device="cuda")
    B.hmy_k_attn_bwd(pc, qd, o, dev(do, dt), lse, delta2, dqkv2, b, s, H, dh, causal, dbias=dbd)
    assert torch.equal(dqkv2, dqkv)
    assert max_rel_err(host(delta2), host(delta)) < 1e-5
    assert max_rel_err(host(delta2).reshape(b, H, s), (do.astype(np.float64) * host(o)).reshape(b, s, H, dh).sum(-1).transpose(0, 2, 1)) < 1e-4
    sums = got.astype(np.float64).sum(axis=0)
    assert np.abs(host(dbd) - db0 - sums).max() < 1e-4 * max(np.abs(sums).max(), np.abs(db0).max(), 1.0)


@pytest.mark.parametrize("prec,pc,dt,tol", PRECS)
@pytest.mark.parametrize("T,V", [(9, 1000), (33, 50257), (4, 2)])
def test_cross_entropy(prec, pc, dt, tol, T, V):
    say(f"xent {prec} T={T} V={V}")
    rng = np.random.default_rng(V)
    ldl = (V + 7) // 8 * 8
    logits = np.zeros((T, ldl), np.float32)
    logits[:, :V] = rng.standard_normal((T, V)).astype(np.float32) * 3
    tg = rng.integers(0, V, size=T).astype(np.int32)
    tg[::3] = -1
    n_tgt = 57                                  # a minibatch-wide count, not this chunk's
    dl = torch.full((T, ldl), float("nan"), device="cuda", dtype=dt)
    acc = torch.zeros(1, device="cuda", dtype=torch.float64)
    B.hmy_k_xent(pc, dev(logits, torch.float32), torch.from_numpy(tg).cuda(), acc, dl, T, V, ldl, 1.0 / n_tgt)
    l64 = logits[:, :V].astype(np.float64)
    lse = np.log(np.exp(l64 - l64.max(1, keepdims=True)).sum(1)) + l64.max(1)
    rows = np.nonzero(tg >= 0)[0]
    loss_ref = (lse[rows] - l64[rows, tg[rows]]).sum() / n_tgt
    assert abs(host(acc)[0] - loss_ref) < 1e-5 * abs(loss_ref)
    ref = np.zeros((T, V))
    ref[rows] = np.exp(l64[rows] - lse[rows, None])
    ref[rows, tg[rows]] -= 1
    ref /= n_tgt
    got = host(dl)
    assert np.all(got[:, V:] == 0)              # the row padding is zeroed
    assert max_rel_err(got[:, :V], ref) < (tol if prec == "bf16" else 1e-5)


@pytest.mark.parametrize("prec,pc,dt,tol", PRECS)
@pytest.mark.parametrize("step", [1, 10])
def test_adam(prec, pc, dt, tol, step):
    say(f"adam {prec} step={step}")
    rng = np.random.default_rng(step)
    n = 4 * 1000 + 3
    w = rng.standard_normal(n).astype(np.float32) * 0.02
    g = rng.standard_normal(n).astype(np.float32) * 1e-3
    m0 = (rng.standard_normal(n).astype(np.float32) * 1e-3) if step > 1 else np.zeros(n, np.float32)
    v0 = ((rng.standard_normal(n).astype(np.float32) * 1e-3) ** 2) if step > 1 else np.zeros(n, np.float32)
    f32 = lambda x: float(np.float32(x))     # the C ABI carries fp32 hyper-parameters
    hp = om.AdamHP(lr=f32(1e-3), beta1=f32(0.9), beta2=f32(0.999), eps=f32(1e-8), step=step)
    wr, mr, vr = om.adam_update(w.astype(np.float64), g.astype(np.float64), m0.astype(np.float64),
                                v0.astype(np.float64), hp)
    gd, md, vd = dev(g, torch.float32), dev(m0, torch.float32), dev(v0, torch.float32)
    if prec == "bf16":
        master = dev(w, torch.float32)
        wout = torch.zeros(n, device="cuda", dtype=torch.bfloat16)
        B.hmy_k_adam(pc, gd, master, md, vd, wout, n, hp.lr, hp.beta1, hp.beta2, hp.eps, step)
        new_master = host(master)
        # the compute copy is exactly the RNE rounding of the fp32 master
        assert np.array_equal(host(wout), synth.round_bf16(new_master.astype(np.float32)).astype(np.float64))
    else:
        wd = dev(w, torch.float32)
        B.hmy_k_adam(pc, gd, None, md, vd, wd, n, hp.lr, hp.beta1, hp.beta2, hp.eps, step)
        new_master = host(wd)
    assert max_rel_err(new_master - w, wr - w) < 1e-4     # the update itself, not w (which barely moves)
    assert max_rel_err(host(md), mr) < 1e-6
    assert max_rel_err(host(vd), vr) < 1e-6
