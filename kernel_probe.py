#!/usr/bin/env python3
"""Run every hot kernel of the iteration on its own, at the shapes of a workload.

    python kernel_probe.py [--config gpt2m] [--reps 20] [--sets 6] [--only "gemm fwd"]

Device tensors only (no pinned host memory, no engine), so the script also runs
under `rocprofv3 --pmc ...`, which is how the per-kernel counters in profiles/ are
collected.  Prints one line per kernel: average launch time from HIP events and
the algorithmic rate (TFLOP/s for contractions, GB/s for streaming kernels).
`--sets` rotates each kernel over that many operand sets so that operands do not
stay cache-resident between launches (1 = hot).
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="gpt2m")
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--sets", type=int, default=6)
    ap.add_argument("--only", default="", help="run only the kernels whose line starts with this text, e.g. 'gemm fwd'")
    ap.add_argument("--pad", type=int, default=0, help="elements added to the leading dimensions of the GEMM operands "
                    "(what strides that are powers of two cost)")
    ap.add_argument("--micro-batch", type=int, default=0, help="sequences per microbatch instead of the configuration's")
    a = ap.parse_args()
    import torch
    from paper_2202_01306_amd import binding as B
    from paper_2202_01306_amd import synth

    if not torch.cuda.is_available():
        print("kernel_probe.py needs a GPU", file=sys.stderr)
        return 3
    cfg = dict(synth.CONFIGS[a.config])
    if a.micro_batch > 0:
        cfg["b"] = a.micro_batch
    if cfg["precision"] != "bf16":
        print("kernel_probe.py times the bf16 kernels; pick a bf16 config", file=sys.stderr)
        return 2
    dt, pc = torch.bfloat16, B.HMY_PREC_BF16
    T, d, f, H, s, V = cfg["b"] * cfg["seq_len"], cfg["d_model"], cfg["d_ffn"], cfg["n_heads"], cfg["seq_len"], cfg["vocab"]
    dh, R = d // H, 512                      # R: rows of one vocabulary-projection chunk
    ldl = (V + 63) // 64 * 64
    n = max(1, a.sets)
    g = torch.Generator(device="cuda").manual_seed(0)

    def rnd(*shape, scale=1.0, dtype=dt):
        return (torch.randn(*shape, device="cuda", generator=g) * scale).to(dtype)

    def timed(name, fns, work, unit):
        if not name.startswith(a.only):
            return
        for fn in fns:
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(a.reps):
            fns[i % len(fns)]()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / a.reps * 1e3
        rate = work / (us * 1e-6) / (1e12 if unit == "TFLOP/s" else 1e9)
        print(f"{name:44s} {us:9.1f} us  {rate:9.1f} {unit}", flush=True)

    def gemm(name, M, N, K, ta, tb, acc=False, bias=False, res=False, gelu=False, lda=None, ldb=None, ldc=None, c32=False):
        if not name.startswith(a.only):
            return
        lda = (lda or (M if ta else K)) + a.pad
        ldb = (ldb or (N if tb else K)) + a.pad
        ldc = ldc or N
        As = [rnd(K if ta else M, lda, scale=0.5) for _ in range(n)]
        Bs = [rnd(K if tb else N, ldb, scale=0.02) for _ in range(n)]
        # a residual is the fp32 residual stream: the output is fp32 too
        Cs = [torch.zeros(M, ldc, device="cuda", dtype=torch.float32 if acc or c32 or res else dt) for _ in range(n)]
        bs = rnd(N) if bias else None
        rs = [rnd(M, N, dtype=torch.float32) for _ in range(n)] if res else None
        gs = [torch.empty(M, N, device="cuda", dtype=dt) for _ in range(n)] if gelu else None
        fns = [(lambda i=i: B.hmy_k_gemm(pc, M, N, K, As[i], lda, Bs[i], ldb, Cs[i], ldc, ta=ta, tb=tb,
                                         c_fp32=int(acc or c32 or res), accumulate=int(acc), bias=bs,
                                         res=rs[i] if res else None, ldr=N if res else 0, res_fp32=int(res),
                                         gelu_out=gs[i] if gelu else None)) for i in range(n)]
        timed(name, fns, 2.0 * M * N * K, "TFLOP/s")

    print(f"# {a.config}: T={T} d={d} f={f} heads={H} seq={s} vocab={V}; {n} operand set(s), {a.reps} launches each")
    gemm("gemm fwd  qkv    [T,3d] = a Wqkv^T + b", T, 3 * d, d, 0, 0, bias=True)
    gemm("gemm fwd  out    [T,d]  = o Wo^T + b + x", T, d, d, 0, 0, bias=True, res=True)
    gemm("gemm fwd  ffn1   [T,f]  = h W1^T + b, gelu", T, f, d, 0, 0, bias=True, gelu=True)
    gemm("gemm fwd  ffn2   [T,d]  = g W2^T + b + x", T, d, f, 0, 0, bias=True, res=True)
    gemm("gemm fwd  logits [R,V]  = z Wh^T (fp32 out)", R, V, d, 0, 0, ldc=ldl, c32=True)
    gemm("gemm dgrad ffn2  [T,f]  = dy W2", T, f, d, 0, 1)
    gemm("gemm dgrad ffn1  [T,d]  = du W1", T, d, f, 0, 1)
    gemm("gemm dgrad out   [T,d]  = dy Wo", T, d, d, 0, 1)
    gemm("gemm dgrad qkv   [T,d]  = dqkv Wqkv", T, d, 3 * d, 0, 1)
    gemm("gemm dgrad head  [T,d] += dlogits Wh", T, d, V, 0, 1, acc=True, lda=ldl)
    gemm("gemm wgrad ffn2  [d,f] += dy^T g", d, f, T, 1, 1, acc=True)
    gemm("gemm wgrad ffn1  [f,d] += du^T h", f, d, T, 1, 1, acc=True)
    gemm("gemm wgrad out   [d,d] += dy^T o", d, d, T, 1, 1, acc=True)
    gemm("gemm wgrad qkv   [3d,d] += dqkv^T a", 3 * d, d, T, 1, 1, acc=True)
    gemm("gemm wgrad head  [V,d] += dlogits^T z", V, d, T, 1, 1, acc=True, lda=ldl)

    b = cfg["b"]
    causal = int(cfg["causal"])
    att_flops = b * H * 4.0 * s * s * dh / (2 if causal else 1)
    qkv = [rnd(T, 3 * d) for _ in range(n)]
    o = [torch.empty(T, d, device="cuda", dtype=dt) for _ in range(n)]
    lse = [torch.empty(b * H * s, device="cuda") for _ in range(n)]
    timed("attention forward", [(lambda i=i: B.hmy_k_attn_fwd(pc, qkv[i], o[i], lse[i], b, s, H, dh, causal)) for i in range(n)],
          att_flops, "TFLOP/s")
    do = [rnd(T, d) for _ in range(n)]
    delta = torch.empty(b * H * s, device="cuda")
    dqkv = torch.empty(T, 3 * d, device="cuda", dtype=dt)
    timed("attention backward (dQ with delta, dK/dV)",
          [(lambda i=i: B.hmy_k_attn_bwd(pc, qkv[i], o[i], do[i], lse[i], delta, dqkv, b, s, H, dh, causal)) for i in range(n)],
          2.5 * att_flops, "TFLOP/s")
    dbias = torch.zeros(3 * d, device="cuda")
    timed("attention backward with the QKV bias gradient",
          [(lambda i=i: B.hmy_k_attn_bwd(pc, qkv[i], o[i], do[i], lse[i], delta, dqkv, b, s, H, dh, causal, dbias=dbias))
           for i in range(n)], 2.5 * att_flops, "TFLOP/s")

    x = [rnd(T, d, dtype=torch.float32) for _ in range(n)]      # the residual stream is fp32
    dy = [rnd(T, d) for _ in range(n)]
    gam, bet = torch.ones(d, device="cuda", dtype=dt), torch.zeros(d, device="cuda", dtype=dt)
    y = torch.empty(T, d, device="cuda", dtype=dt)
    mean, rstd = torch.empty(T, device="cuda"), torch.empty(T, device="cuda")
    timed("layernorm forward", [(lambda i=i: B.hmy_k_layernorm_fwd(pc, x[i], gam, bet, y, mean, rstd, T, d, synth.LN_EPS)) for i in range(n)],
          T * d * (4.0 + 2.0), "GB/s")
    dgm, dbt = torch.zeros(d, device="cuda"), torch.zeros(d, device="cuda")
    ws = torch.empty(256 * 3 * d, device="cuda")
    dx32 = torch.empty(T, d, device="cuda")
    dbias = torch.zeros(d, device="cuda")
    timed("layernorm backward (+ bias gradient, + partial-sum reduce)",
          [(lambda i=i: B.hmy_k_layernorm_bwd(pc, dy[i], x[i], mean, rstd, gam, x[(i + 1) % n], dx32, dgm, dbt, T, d, workspace=ws,
                                              dx_e=y, dres_sum=dbias))
           for i in range(n)], T * d * (2.0 + 4 + 4 + 4 + 2), "GB/s")     # dy, x, res in; dx (fp32) and its bf16 copy out
    timed("layernorm backward (+ bias gradient), sums by atomics",
          [(lambda i=i: B.hmy_k_layernorm_bwd(pc, dy[i], x[i], mean, rstd, gam, x[(i + 1) % n], dx32, dgm, dbt, T, d, dx_e=y,
                                              dres_sum=dbias))
           for i in range(n)], T * d * (2.0 + 4 + 4 + 4 + 2), "GB/s")
    u = [rnd(T, f) for _ in range(n)]
    dg = [rnd(T, f) for _ in range(n)]
    du = torch.empty(T, f, device="cuda", dtype=dt)
    timed("gelu backward", [(lambda i=i: B.hmy_k_gelu_bwd(pc, dg[i], u[i], du, T * f)) for i in range(n)], 3.0 * T * f * 2, "GB/s")
    db1 = torch.zeros(f, device="cuda")
    timed("gelu backward + bias gradient", [(lambda i=i: B.hmy_k_gelu_bwd_colsum(pc, dg[i], u[i], du, db1, T, f)) for i in range(n)],
          3.0 * T * f * 2, "GB/s")
    for N in (d, 3 * d, f):
        out = torch.zeros(N, device="cuda")
        src = u if N == f else [rnd(T, N) for _ in range(n)]
        timed(f"column sums [T,{N}]", [(lambda i=i: B.hmy_k_colsum(pc, src[i], out, T, N)) for i in range(n)], 1.0 * T * N * 2, "GB/s")
    logits = [rnd(R, ldl, dtype=torch.float32) for _ in range(min(n, 3))]
    tg = torch.randint(0, V, (R,), device="cuda", dtype=torch.int32)
    loss = torch.zeros(1, device="cuda", dtype=torch.float64)
    dl = torch.empty(R, ldl, device="cuda", dtype=dt)
    timed("softmax cross-entropy [R,V] (2 reads from HBM/L2)",
          [(lambda i=i: B.hmy_k_xent(pc, logits[i], tg, loss, dl, R, V, ldl, 1.0 / R)) for i in range(len(logits))],
          R * (2.0 * V * 4 + V * 2), "GB/s")
    P = 4 << 20
    grad, mst, m1, v1 = (torch.zeros(P, device="cuda") for _ in range(4))
    w = torch.empty(P, device="cuda", dtype=dt)
    timed("adam (HBM-resident state, 30 B/param)", [lambda: B.hmy_k_adam(pc, grad, mst, m1, v1, w, P, 1e-4, 0.9, 0.999, 1e-8, 2)],
          30.0 * P, "GB/s")
    return 0


if __name__ == "__main__":
    sys.exit(main())
