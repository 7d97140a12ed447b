#!/usr/bin/env python3
"""Benchmark: one layer-pack-major training iteration under the HBM budget.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config gpt2m] [--no-cpu-baseline]

A step is one whole iteration (every forward pack, the last pack's
forward+backward, every backward pack with recompute, fused Adam and all swaps)
on synthetic data with model state starting in pinned host memory, which is
where the method keeps it.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
HOST_LINK_GBPS_ALONE = 54.0    # pinned host <-> HBM, one direction, nothing else running (measured on the GPU machine)
PEAK_FP32_TFLOPS = 157.3
VARIANTS = ("gemm_mfma<A[M,K],B[N,K]> (forward, recompute)", "gemm_mfma<A[M,K],B[K,N]> (input gradient)",
            "gemm_mfma<A[K,M],B[N,K]>", "gemm_mfma<A[K,M],B[K,N]> (weight gradient)")


def attention_flops(cfg, packs) -> float:
    """Algorithmic attention flops of one iteration: QK^T and PV forward (causal
    counts the visible half), 2.5x that for backward, forward repeated once for
    every block that is recomputed (all but the last backward pack)."""
    P_F, P_B = packs
    L, s, d = cfg["n_blocks"], cfg["seq_len"], cfg["d_model"]
    tokens = cfg["M"] * cfg["b"] * s
    fwd = tokens * (2 if cfg["causal"] else 4) * s * d
    last_a = P_B[-1][0]
    recomputed = sum(1 for l in range(1, L + 1) if l < last_a)
    return fwd * (L + recomputed) + 2.5 * fwd * L


# HBM traffic of the forward-variant GEMM launches of one gpt2m iteration: FETCH_SIZE and WRITE_SIZE (KiB per
# dispatch, averaged per kernel and grid) from two `rocprofv3 --pmc` runs over `bench.py --counters`, i.e. over the
# launches of a real iteration.  Copied from profiles/gpt2m_forward_gemm_hbm_traffic.md, which has the commands; kept
# here because counters cannot be collected inside the timed run itself.  FETCH_SIZE is scaled by 2.0 and
# WRITE_SIZE by 1.0: what the same counters read for a streaming kernel of known size (k_gelu_bwd_colsum, 64 MiB in /
# 32 MiB plus 4 MiB of atomic additions out).
GPT2M_FWD_GEMM_TRAFFIC = [   # (what, kernel, grid threads, dispatches, FETCH_SIZE KiB as counted, WRITE_SIZE KiB)
    ("ffn1", "k_gemm_dma256<false, false, 64, 2>", 131072, 384, 24924.5, 49152.0),
    ("qkv", "k_gemm_dma256<false, false, 64, 2>", 98304, 384, 20820.5, 24576.0),
    ("logits, 512-row chunk", "k_gemm_dma256<false, false, 64, 2>", 201728, 64, 60320.8, 100528.1),
    ("out and ffn2", "k_gemm_dma<false, false, 64, 4>", 65536, 704, 37451.9, 16384.0),
]


def nt_gemm_traffic_per_launch(config_name, cfg, packs, nt_calls):
    """(measured, algorithmic) average HBM bytes per launch of the forward-variant GEMM over one
    iteration, or None where no counters were collected for the workload's shapes."""
    if config_name != "gpt2m":
        return None
    measured = (sum(n * (2.0 * f + w) * 1024 for (_, _, _, n, f, w) in GPT2M_FWD_GEMM_TRAFFIC)
                / sum(n for (_, _, _, n, _, _) in GPT2M_FWD_GEMM_TRAFFIC))
    # what the launches of THIS run must move at least: each operand and result once (bf16; the residual stream and
    # the logits fp32); FFN1 writes its pre-activation too where a backward pass will need it
    P_F, P_B = packs
    L, M = cfg["n_blocks"], cfg["M"]
    is_block = lambda layer: 1 <= layer <= L
    last_a, last_e = P_B[-1]
    n_last = sum(1 for l in range(last_a, last_e) if is_block(l))
    block_fwd = M * (2 * L - n_last)                        # forward pass + recompute, last pack once
    kept = M * L                                            # every block once with its activations kept
    # the recompute of a backward pack stops before the FFN2 GEMM of its last block (its output is not needed)
    skipped = M * sum(1 for (a, e) in P_B[:-1] if is_block(e - 1))
    calls = {"qkv": block_fwd, "out": block_fwd, "ffn1_kept": kept, "ffn1": block_fwd - kept,
             "ffn2": block_fwd - skipped}
    calls["logits"] = nt_calls - sum(calls.values())
    if calls["logits"] < 0:
        return None
    T, d, f, V, R = cfg["b"] * cfg["seq_len"], cfg["d_model"], cfg["d_ffn"], cfg["vocab"], 512
    ldl = (V + 63) // 64 * 64
    algo = {"qkv": 2 * (T * d + 3 * d * d + 3 * d + T * 3 * d), "out": 2 * (T * d + d * d + d) + 8 * T * d,
            "ffn1_kept": 2 * (T * d + f * d + f + 2 * T * f), "ffn1": 2 * (T * d + f * d + f + T * f),
            "ffn2": 2 * (T * f + d * f + d) + 8 * T * d, "logits": 2 * (R * d + V * d) + 4 * R * ldl}
    return measured, sum(calls[k] * algo[k] for k in algo) / nt_calls


def cpu_baseline(cfg):
    """Time the fp64 oracle, as it stands, on a bounded sample of the workload:
    embedding, ONE block and the head, forward and backward, on one microbatch at
    full width; extrapolated linearly to all blocks and microbatches."""
    import numpy as np
    from oracle import model as om
    from paper_2202_01306_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    c1 = dict(cfg, n_blocks=1, M=1)
    spec = om.Spec(1, cfg["d_model"], cfg["n_heads"], cfg["d_ffn"], cfg["seq_len"], cfg["vocab"], bool(cfg["causal"]),
                   synth.LN_EPS)
    params = {k: np.asarray(v, np.float64) for k, v in synth.gen_params(c1, 0).items()}
    ids = synth.gen_tokens(c1, 0)
    tg = synth.gen_targets(c1, ids, 0)
    n_tgt = om.count_targets(tg)
    t = {}
    x, caches = None, []
    for layer in range(3):
        t0 = time.perf_counter()
        x, c = om.layer_fwd(layer, x, params, spec, ids[0], tg[0], n_tgt)
        t[("f", layer)] = time.perf_counter() - t0
        caches.append(c)
    dy = None
    for layer in (2, 1, 0):
        t0 = time.perf_counter()
        dy, _ = om.layer_bwd(layer, dy, caches[layer], params, spec, cfg["b"])
        t[("b", layer)] = time.perf_counter() - t0
    t_block = t[("f", 1)] + t[("b", 1)]
    t_rest = t[("f", 0)] + t[("b", 0)] + t[("f", 2)] + t[("b", 2)]
    est = cfg["M"] * (cfg["n_blocks"] * t_block + t_rest)
    return {
        "value": cfg["M"] * cfg["b"] / est, "unit": "samples/s", "cores": int(cores), "kind": "oracle",
        "sample": (f"fp64 numpy oracle: embedding + 1 block + head, forward+backward, 1 microbatch of "
                   f"{cfg['b']}x{cfg['seq_len']} tokens at full width ({sum(t.values()):.1f} s of CPU work; block "
                   f"{t_block:.2f} s, embedding+head {t_rest:.2f} s), extrapolated linearly to "
                   f"{cfg['n_blocks']} blocks x {cfg['M']} microbatches (no recompute, no swapping)"),
    }


def measured_profiles(B, spec, sizes, reps=10):
    """The Profiler step (Section 4.2): per-layer times of this library's kernels on the device, one entry per
    microbatch size the planner may consider."""
    return [B.hmy_measure_profile(spec, u, reps=reps) for u in sizes]


def plan_kwargs(a, measured):
    """What the planner may sweep in this run (binding.make_budget)."""
    kw = dict(search=a.pack_search, slots=(a.min_slots, a.max_slots))
    if measured:
        kw["measured"] = measured
    return kw


def step_bound(total_flops, h2d, d2h, ms, peak):
    """The step against what bounds it from below: all of its flops at the MFMA peak, or the busier direction of
    the host link at the rate the link gives with the device otherwise idle (measured, 54 GB/s)."""
    mfma_s, link_s = total_flops / (peak * 1e12), max(h2d, d2h) / (HOST_LINK_GBPS_ALONE * 1e9)
    return {"mfma_ms": mfma_s * 1e3, "host_link_ms": link_s * 1e3, "host_link_GBps_alone": HOST_LINK_GBPS_ALONE,
            "frac": max(mfma_s, link_s) / (ms * 1e-3)}


def run_other_workload(B, synth, Engine, TrainingState, name, a, steps=2, update_site="device"):
    """A short run of another of the named workloads, planned the same way: its own measured profile, packs,
    time per step, swap volumes and bounds.  Returns a dict for the JSON line, or one that says why it did not run."""
    cfg = dict(synth.CONFIGS[name])
    host = update_site == "host"
    try:
        st = TrainingState(cfg, pageable_optimizer_state=host)
    except (B.HmyError, MemoryError) as e:
        return {"skipped": f"cannot hold the host state on this box: {e}"}
    try:
        st.fill_random(0, tile=1 << 27)
        ids = synth.gen_tokens(cfg, 0)
        tg = synth.gen_targets(cfg, ids, 0)
        meas = None if a.analytic_profile else measured_profiles(B, st.spec, [cfg["b"]])
        site = B.HMY_UPDATE_ON_HOST if host else B.HMY_UPDATE_ON_DEVICE
        try:
            eng = Engine(st, cfg["budget"], cfg["M"], cfg["b"], update_site=site, **plan_kwargs(a, meas))
        except B.HmyError as e:
            return {"skipped": f"engine: {e}"}
        with eng:
            eng.set_batch(ids, tg)
            eng.step(step=1, want_stats=False)
            t0 = time.perf_counter()
            for i in range(steps):
                stats = eng.step(step=2 + i, want_stats=True)
            ms = (time.perf_counter() - t0) / steps * 1e3
            B.hmy_set_profiling(eng.handle, 2)
            prof = eng.step(step=2 + steps, want_stats=True)
            packs, arena, sched = eng.packs, eng.arena, eng.sched
            est_ms = B.hmy_estimate(st.spec, sched, cfg["M"], cfg["b"], measured=meas) / 1e6
        peak = PEAK_BF16_TFLOPS if cfg["precision"] == "bf16" else PEAK_FP32_TFLOPS
        h2d, d2h = sum(stats["h2d"].values()), sum(stats["d2h"].values())
        flops = sum(prof["gemm_flops"]) + attention_flops(cfg, packs)
        return {"workload": f"{name}: {cfg['n_blocks']} blocks d={cfg['d_model']} heads={cfg['n_heads']} ffn={cfg['d_ffn']} "
                            f"seq={cfg['seq_len']} vocab={cfg['vocab']}, {cfg['M']} microbatches x {cfg['b']} sequences",
                "hbm_budget_bytes": cfg["budget"], "arena_bytes": arena["total"], "update_site": update_site,
                "optimizer_state_memory": "pageable" if host else "pinned",
                "weight_slots": arena["weight_slots"], "prefetch_distance": arena["prefetch_distance"],
                "fwd_packs": packs[0], "bwd_packs": packs[1], "steps": steps,
                "value": cfg["M"] * cfg["b"] / (ms * 1e-3), "unit": "samples/s", "ms_per_step": ms,
                "planner_estimate_ms": est_ms, "estimate_over_measured": est_ms / ms,
                "tflops": flops / (ms * 1e-3) / 1e12,
                "gemm_variants_TFLOPs": [prof["gemm_flops"][i] / max(prof["gemm_s"][i], 1e-12) / 1e12
                                         if prof["gemm_calls"][i] else None for i in range(4)],
                "h2d_GB_per_iter": h2d / 1e9, "d2h_GB_per_iter": d2h / 1e9, "loss": stats["loss"],
                "step_bound": step_bound(flops, h2d, d2h, ms, peak)}
    finally:
        st.close()


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="gpt2m")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pack-search", type=int, default=None,
                    help="how many pack counts beyond the first feasible one the planner may try (0 = Algorithm 2 alone)")
    ap.add_argument("--min-slots", type=int, default=2, help="fewest weight slots the planner may choose")
    ap.add_argument("--max-slots", type=int, default=4, help="most weight slots the planner may choose")
    ap.add_argument("--analytic-profile", action="store_true",
                    help="plan from flop counts over one sustained rate instead of per-layer times measured at start-up")
    ap.add_argument("--reference-kernels", action="store_true", help="time the plain (non-MFMA) kernels")
    ap.add_argument("--order", choices=("layer-pack-major", "microbatch-major"), default="layer-pack-major",
                    help="microbatch-major: the order the paper compares against, over the same packs (ablation)")
    ap.add_argument("--gradients", choices=("exported", "device"), default="exported",
                    help="device: the update drops the gradient it consumed, as in the paper (no dW on the link)")
    ap.add_argument("--resident-state", action="store_true",
                    help="keep optimizer state on the device in what the budget leaves free behind the arena")
    ap.add_argument("--no-variants", action="store_true",
                    help="skip the extra short runs reported under 'variants' and 'other_workloads'")
    ap.add_argument("--update-site", choices=("device", "host"), default="device",
                    help="host: the Weight Update task runs on CPU threads (the paper's optimizer offload); "
                         "optimizer state then never crosses the link")
    ap.add_argument("--fwd-packs", default="", help="forward pack ends instead of the planner's, e.g. 2,6,14,25 "
                    "(the last backward pack's first layer closes the list)")
    ap.add_argument("--bwd-packs", default="", help="backward pack ends instead of the planner's, e.g. 1,3,7,26")
    ap.add_argument("--slots", type=int, default=0, help="weight slots instead of the planner's choice")
    ap.add_argument("--distance", type=int, default=0, help="prefetch distance instead of the planner's choice")
    ap.add_argument("--counters", action="store_true",
                    help="for runs under `rocprofv3 --pmc`, where every dispatch is serialised: ONE iteration, no warm-up, "
                         "no variants, no CPU baseline, and a line on stderr after every visit")
    a = ap.parse_args()
    if a.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus {a.gpus} is not supported",
              file=sys.stderr)
        return 2
    if a.counters:
        a.steps, a.warmup, a.no_variants, a.no_cpu_baseline, a.analytic_profile = 1, 0, True, True, True

    # No PyTorch in this process: the library then runs on the HIP runtime it was
    # linked against (ROCm's own), not on the older copy bundled with the wheel.
    from paper_2202_01306_amd import binding as B
    from paper_2202_01306_amd import synth
    from paper_2202_01306_amd.runner import Engine, TrainingState

    if a.pack_search is None:
        from paper_2202_01306_amd.runner import BENCH_PACK_SEARCH
        a.pack_search = BENCH_PACK_SEARCH
    cfg = dict(synth.CONFIGS[a.config])
    if cfg["budget"] is None:
        cfg["budget"] = 1 << 30
    if a.reference_kernels:
        B.hmy_set_kernel_path(False)
    try:
        st = TrainingState(cfg)        # pinned host memory: the first call that needs the GPU
    except B.HmyError as e:
        if a.update_site == "host" and "out of memory" in str(e):
            # more state than this machine will page-lock: with the update on the host only CPU threads touch
            # master, m and v, which may then be ordinary memory
            st = TrainingState(cfg, pageable_optimizer_state=True)
        else:
            print(f"bench.py needs a GPU (there is no CPU fallback): {e}", file=sys.stderr)
            return 3
    st.fill_random(0)
    ids = synth.gen_tokens(cfg, 0)
    tg = synth.gen_targets(cfg, ids, 0)
    D = cfg["M"] * cfg["b"]
    # the Profiler step: this library's kernels timed per layer, for the caller's microbatch size and the ones
    # the configuration search of the 'configuration_search' variant may pick instead
    sweep_sizes = sorted({u for u in (cfg["b"] // 2, cfg["b"], 2 * cfg["b"]) if u >= 1 and D % u == 0})
    measured = None if (a.analytic_profile or a.reference_kernels) else measured_profiles(B, st.spec, sweep_sizes)
    site = B.HMY_UPDATE_ON_HOST if a.update_site == "host" else B.HMY_UPDATE_ON_DEVICE
    pkw = plan_kwargs(a, measured)
    sched = B.hmy_plan(st.spec, cfg["budget"], cfg["M"], cfg["b"], update_site=site, **pkw)
    for given, n_field, end_field in ((a.fwd_packs, "n_fwd_packs", "fwd_pack_end"), (a.bwd_packs, "n_bwd_packs", "bwd_pack_end")):
        if given:   # the caller's packs; hmy_create rejects them if they do not fit the budget
            ends = [int(x) for x in given.split(",")]
            setattr(sched, n_field, len(ends))
            for i, e in enumerate(ends):
                getattr(sched, end_field)[i] = e
    if a.slots:
        sched.weight_slots = a.slots
    if a.distance:
        sched.prefetch_distance = a.distance
    sched.order = B.HMY_ORDER_MICROBATCH_MAJOR if a.order == "microbatch-major" else B.HMY_ORDER_LAYER_PACK_MAJOR
    sched.gradients = B.HMY_GRADIENTS_ON_DEVICE if a.gradients == "device" else B.HMY_GRADIENTS_EXPORTED
    sched.resident_state = B.HMY_STATE_RESIDENT_IN_SPARE_BUDGET if a.resident_state else B.HMY_STATE_SWAPPED
    estimate_ms = B.hmy_estimate(st.spec, sched, cfg["M"], cfg["b"], measured=measured) / 1e6
    with Engine(st, cfg["budget"], cfg["M"], cfg["b"], sched) as eng:
        eng.set_batch(ids, tg)
        step = 1
        if a.counters:
            B.hmy_set_progress(eng.handle, True)
        for _ in range(a.warmup):
            eng.step(step=step, want_stats=False)
            step += 1
        t0 = time.perf_counter()                           # every step returns with all streams idle
        for _ in range(a.steps):
            stats = eng.step(step=step, want_stats=True)   # profiling level 0: byte counters and loss only
            step += 1
        dt = time.perf_counter() - t0
        prof = stats
        if not a.counters:
            # two more identical steps outside the timed region: one with events around every copy and every
            # wait of the compute stream (link rates, stall, hidden fraction), one with events around every
            # GEMM launch as well (the roofline block); the events themselves cost a few percent
            B.hmy_set_profiling(eng.handle, 1)
            stats = eng.step(step=step, want_stats=True)
            step += 1
            B.hmy_set_profiling(eng.handle, 2)
            prof = eng.step(step=step, want_stats=True)
            step += 1
            B.hmy_set_profiling(eng.handle, 0)
        packs, arena, resident = eng.packs, eng.arena, eng.resident_params()
        eng.sync_state()

    # Variants outside the timed region of the headline number: the paper's optimizer offload (Weight Update on
    # CPU threads), the paper's own dW traffic (none: the update drops the gradient it consumed instead of
    # exporting it), optimizer state kept on the device in what the budget leaves free behind the arena (then
    # the host arrays hold that state only after hmy_sync_state), both, the configuration search of Algorithm 1
    # free to choose another microbatch size per pass, and the order the method is compared against.
    variants = {}
    others = {}
    if not a.no_variants and a.order == "layer-pack-major" and a.update_site == "device" and not a.reference_kernels:
        LPM, MBM = B.HMY_ORDER_LAYER_PACK_MAJOR, B.HMY_ORDER_MICROBATCH_MAJOR
        DEV, HOST = B.HMY_UPDATE_ON_DEVICE, B.HMY_UPDATE_ON_HOST
        SWAP, RES = B.HMY_STATE_SWAPPED, B.HMY_STATE_RESIDENT_IN_SPARE_BUDGET
        EXP, DROP = B.HMY_GRADIENTS_EXPORTED, B.HMY_GRADIENTS_ON_DEVICE
        for name, order, vsite, grads, res, n, sweep in (
                ("update_on_host", LPM, HOST, EXP, SWAP, max(2, a.steps), False),
                ("gradients_on_device", LPM, DEV, DROP, SWAP, max(2, a.steps), False),
                ("resident_state", LPM, DEV, EXP, RES, max(2, a.steps), False),
                ("resident_state+gradients_on_device", LPM, DEV, DROP, RES, max(2, a.steps), False),
                ("configuration_search", LPM, DEV, EXP, SWAP, max(2, a.steps), True),
                ("microbatch_major", MBM, DEV, EXP, SWAP, 2, False)):
            if (grads == DROP) == (a.gradients == "device") and (res == RES) == a.resident_state and order == LPM \
                    and vsite == DEV and not sweep:
                continue    # that is the headline run itself
            # the host variant over the packs the planner picks for it (its estimate knows that only the
            # gradient crosses the link then); the others over the headline's packs
            kw = dict(pkw)
            if sweep:
                kw.update(max_fwd_micro_batch=sweep_sizes[-1], max_bwd_micro_batch=sweep_sizes[-1])
            vs = B.hmy_plan(st.spec, cfg["budget"], cfg["M"], cfg["b"], update_site=vsite, **kw)
            vs.order, vs.gradients, vs.resident_state = order, grads, res
            vest = B.hmy_estimate(st.spec, vs, cfg["M"], cfg["b"], measured=measured) / 1e6
            with Engine(st, cfg["budget"], cfg["M"], cfg["b"], vs) as eng:
                eng.set_batch(ids, tg)
                eng.step(step=step, want_stats=False)
                step += 1
                t0 = time.perf_counter()
                for _ in range(n):
                    vstats = eng.step(step=step, want_stats=True)
                    step += 1
                vms = (time.perf_counter() - t0) / n * 1e3
                vpacks, vres, varena = eng.packs, eng.resident_params(), eng.arena
                eng.sync_state()      # the next variant starts from complete host arrays
            variants[name] = {"fwd_packs": vpacks[0], "bwd_packs": vpacks[1], "resident_state_params": vres,
                              "weight_slots": varena["weight_slots"], "prefetch_distance": varena["prefetch_distance"],
                              "fwd_micro_batch": varena["fwd_micro_batch"], "bwd_micro_batch": varena["bwd_micro_batch"],
                              "value": cfg["M"] * cfg["b"] / (vms * 1e-3), "unit": "samples/s", "ms_per_step": vms, "steps": n,
                              "planner_estimate_ms": None if (order == MBM or res == RES) else vest,
                              "h2d_GB_per_iter": sum(vstats["h2d"].values()) / 1e9,
                              "d2h_GB_per_iter": sum(vstats["d2h"].values()) / 1e9}
    st.close()      # page-locked memory back before the other workloads take theirs
    if not a.no_variants and a.config == "gpt2m" and a.order == "layer-pack-major" and a.update_site == "device" \
            and not a.reference_kernels:
        # the other named workloads, two steps each: the encoder (compute-bound), the 1.5 B decoder, and the
        # 6.7 B decoder whole with the update on the host (124 GB of page-locked state does not fit this box;
        # with the optimizer on the CPU only weights and gradients need locking)
        others["bertl"] = run_other_workload(B, synth, Engine, TrainingState, "bertl", a)
        others["gpt2xl"] = run_other_workload(B, synth, Engine, TrainingState, "gpt2xl", a)
        others["gpt6b7_update_on_host"] = run_other_workload(B, synth, Engine, TrainingState, "gpt6b7", a,
                                                             update_site="host")

    ms = dt / a.steps * 1e3
    samples = cfg["M"] * cfg["b"]
    gemm_flops = sum(prof["gemm_flops"])
    gemm_s = sum(prof["gemm_s"])
    dom = max(range(4), key=lambda i: prof["gemm_s"][i])
    peak = PEAK_BF16_TFLOPS if cfg["precision"] == "bf16" else PEAK_FP32_TFLOPS
    dom_tflops = prof["gemm_flops"][dom] / max(prof["gemm_s"][dom], 1e-12) / 1e12
    h2d = sum(stats["h2d"].values())
    d2h = sum(stats["d2h"].values())
    copy_s = stats["t_h2d_busy_s"] + stats["t_d2h_busy_s"]
    total_flops = gemm_flops + attention_flops(cfg, packs)
    traffic = nt_gemm_traffic_per_launch(a.config, cfg, packs, prof["gemm_calls"][0]) if dom == 0 else None
    out = {
        "metric": "samples/sec per iteration under HBM budget; swap GB/iter; MFMA util %",
        "value": samples / (ms * 1e-3), "unit": "samples/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["precision"], "data": "synthetic",
        "config": {"workload": f"{a.config}: {cfg['n_blocks']} blocks d={cfg['d_model']} heads={cfg['n_heads']} "
                               f"ffn={cfg['d_ffn']} seq={cfg['seq_len']} vocab={cfg['vocab']}, "
                               f"{cfg['M']} microbatches x {cfg['b']} sequences",
                   "hbm_budget_bytes": cfg["budget"], "arena_bytes": arena["total"],
                   "order": a.order, "update_site": a.update_site, "gradients": a.gradients, "resident_state_params": resident,
                   "fwd_packs": packs[0], "bwd_packs": packs[1], "pack_search": a.pack_search,
                   "weight_slots": arena["weight_slots"], "prefetch_distance": arena["prefetch_distance"],
                   "weight_slots_swept": [a.min_slots, a.max_slots],
                   "fwd_micro_batch": arena["fwd_micro_batch"], "bwd_micro_batch": arena["bwd_micro_batch"],
                   "profile": "measured per layer at start-up" if measured else "flops over one sustained rate",
                   "measured_profile_ns": measured,
                   "planner_estimate_ms": estimate_ms, "estimate_over_measured": estimate_ms / ms,
                   "kernels": "reference" if a.reference_kernels else "mfma"},
        "tflops": total_flops / (ms * 1e-3) / 1e12,
        "swap": {"h2d_GB_per_iter": h2d / 1e9, "d2h_GB_per_iter": d2h / 1e9,
                 "h2d_by_kind_GB": {k: v / 1e9 for k, v in stats["h2d"].items() if v},
                 "d2h_by_kind_GB": {k: v / 1e9 for k, v in stats["d2h"].items() if v},
                 "h2d_GBps_while_copying": h2d / 1e9 / max(stats["t_h2d_busy_s"], 1e-12),
                 "d2h_GBps_while_copying": d2h / 1e9 / max(stats["t_d2h_busy_s"], 1e-12),
                 "compute_stall_s": stats["t_stall_s"],
                 "hidden_fraction": 1.0 - stats["t_stall_s"] / max(copy_s, 1e-12)},
        "timeline_ms": {"note": "one extra step with timing events on every copy and wait (slower than ms_per_step)",
                        "iteration_host_clock": stats["t_iter_s"] * 1e3,
                        "compute_stream_first_to_last_kernel": stats["t_compute_s"] * 1e3,
                        "compute_stream_waiting_on_swaps": stats["t_stall_s"] * 1e3,
                        "outside_compute_span(prologue+epilogue)": (stats["t_iter_s"] - stats["t_compute_s"]) * 1e3,
                        "h2d_copy_busy": stats["t_h2d_busy_s"] * 1e3, "d2h_copy_busy": stats["t_d2h_busy_s"] * 1e3},
        "mfma_util_pct": 100.0 * gemm_flops / max(gemm_s, 1e-12) / 1e12 / peak,
        "roofline": {"bound": "mfma", "kernel": VARIANTS[dom], "achieved": dom_tflops, "peak": peak,
                     "unit": "TFLOP/s", "frac": dom_tflops / peak,
                     "traffic": traffic[0] if traffic else None,
                     "traffic_unit": "HBM bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated; stored, not live: "
                                     "profiles/gpt2m_forward_gemm_hbm_traffic.md)",
                     "algorithmic_bytes_per_launch": traffic[1] if traffic else None,
                     "launches": prof["gemm_calls"][dom],
                     "avg_launch_us": prof["gemm_s"][dom] / max(prof["gemm_calls"][dom], 1) * 1e6,
                     "event_pair_us_subtracted_per_launch": prof["t_event_pair_s"] * 1e6,
                     "all_variants_TFLOPs": [prof["gemm_flops"][i] / max(prof["gemm_s"][i], 1e-12) / 1e12
                                             if prof["gemm_calls"][i] else None for i in range(4)]},
        # the kernels that write to the host (fused Adam + write-back, checkpoint copies) own the other stream:
        # bytes they moved over the time they ran (events of the level-1 step) against the link alone
        "roofline_host_link": {"bound": "host_link", "kernel": "k_adam_out + k_copy_out (device->host)",
                               "achieved": d2h / 1e9 / max(stats["t_d2h_busy_s"], 1e-12), "peak": HOST_LINK_GBPS_ALONE,
                               "unit": "GB/s", "frac": d2h / 1e9 / max(stats["t_d2h_busy_s"], 1e-12) / HOST_LINK_GBPS_ALONE,
                               "busy_ms": stats["t_d2h_busy_s"] * 1e3,
                               "note": "peak = what the same kernels reach with nothing else running (measured); "
                                       "throttled on purpose beside the compute stream"},
        "step_bound": step_bound(total_flops, h2d, d2h, ms, peak),
        "loss": stats["loss"],
    }
    if variants:
        out["variants"] = variants
    if others:
        out["other_workloads"] = others
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
