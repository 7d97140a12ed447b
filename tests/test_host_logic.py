"""CPU tests of the C-ABI library's host logic against the oracle: exported
symbols, tensor layout, analytic profile, Algorithm 2 planner, arena sizing and
the swap-byte counters of a dry walk of the executor (bit-exact)."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import model as om
from oracle import packing as opk
from oracle import swapcount as osw
from paper_2202_01306_amd import binding as B
from paper_2202_01306_amd import synth
from tests.helpers import oracle_spec, tiny_cfg
from tests.test_oracle_schedule import all_packings

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "hmy.h")).read()
    declared = set(re.findall(r"^(?:int|const char \*)\s*(hmy_[a-z0-9_]+)\s*\(", hdr, flags=re.M))
    assert len(declared) >= 28
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(B.lib, name), name
        getattr(B.lib, name)


def test_struct_sizes_match_what_a_c_compiler_gives_for_the_header(tmp_path):
    """The header must be valid C, and the ctypes mirrors must agree with it."""
    import subprocess
    names = ["hmy_model_spec", "hmy_budget", "hmy_schedule", "hmy_minibatch", "hmy_adam", "hmy_host_state",
             "hmy_stats", "hmy_tensor_desc", "hmy_layer_profile", "hmy_arena_plan", "hmy_gemm_desc",
             "hmy_measured_profile", "hmy_region"]
    src = tmp_path / "sz.c"
    src.write_text('#include <stdio.h>\n#include "hmy.h"\nint main(void){' +
                   "".join(f'printf("%zu\\n", sizeof({n}));' for n in names) +
                   'printf("%d %d\\n", HMY_MAX_LAYERS, HMY_NKINDS);return 0;}')
    exe = tmp_path / "sz"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)],
                   check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    for n, sz in zip(names, out):
        assert ctypes.sizeof(getattr(B, n)) == int(sz), n
    assert (int(out[-2]), int(out[-1])) == (B.HMY_MAX_LAYERS, B.HMY_NKINDS)
    hdr = open(os.path.join(ROOT, "include", "hmy.h")).read()
    assert f"#define HMY_MAX_WEIGHT_SLOTS {B.HMY_MAX_WEIGHT_SLOTS}" in hdr


@pytest.mark.parametrize("name", list(synth.CONFIGS))
def test_layout_matches_the_named_shapes(name):
    cfg = synth.CONFIGS[name]
    spec = B.make_spec(cfg)
    lay = B.hmy_layout(spec)
    shapes = synth.shape_table(cfg)
    assert [t["name"] for t in lay] == list(shapes)
    off = 0
    ospec = oracle_spec(cfg)
    for t, (nm, shp) in zip(lay, shapes.items()):
        assert t["count"] == int(np.prod(shp)) and t["offset"] == off
        assert (t["rows"], t["cols"]) == (shp[0], shp[1] if len(shp) == 2 else 1)
        assert nm in om.layer_param_shapes(ospec, t["layer"])
        off += t["count"]
    R, n = B.hmy_model_size(spec)
    assert R == ospec.n_layers and n == off == sum(om.layer_param_count(ospec, l) for l in range(R))


def _elem(cfg):
    return 2 if cfg["precision"] == "bf16" else 4


@pytest.mark.parametrize("name", list(synth.CONFIGS))
def test_profile_states_the_workload(name):
    """The per-layer profile against what the model's definition fixes: parameter counts are the oracle's; forward
    flops per token of a block are 2 (4 d^2 + 2 d f) for the four linear maps plus 2 s d (causal, masked half not
    counted) or 4 s d for the attention products, of the head 2 d V; a backward task costs three forwards (recompute
    and two products per forward product); times are flops over the given rate, rounded up; the byte footprints are
    the weight (and fp32 gradient) bytes in every slot plus the activations."""
    cfg = synth.CONFIGS[name]
    spec, ospec = B.make_spec(cfg), oracle_spec(cfg)
    d, f, s_, V, T, E = cfg["d_model"], cfg["d_ffn"], cfg["seq_len"], cfg["vocab"], cfg["b"] * cfg["seq_len"], _elem(cfg)
    for slots, rate in ((3, 420000), (2, 1000)):
        prof, res = B.hmy_profile(spec, cfg["M"], cfg["b"], sched=B.make_schedule([], [], slots=slots),
                                  budget=B.make_budget(0, compute_GFLOPs=rate))
        assert len(prof) == ospec.n_layers
        for l, p in enumerate(prof):
            assert p["params"] == om.layer_param_count(ospec, l)
            if 1 <= l <= cfg["n_blocks"]:
                assert p["flops_fwd"] == T * (2 * (4 * d * d + 2 * d * f) + (2 if cfg["causal"] else 4) * s_ * d)
            elif l > cfg["n_blocks"]:
                assert p["flops_fwd"] == 2 * T * d * V
            assert p["ns_fwd"] == -(-p["flops_fwd"] // rate) and p["ns_bwd"] == -(-3 * p["flops_fwd"] // rate)
            assert p["mem_fwd"] == slots * E * p["params"]
            assert p["mem_bwd"] == slots * (E + 4) * p["params"] + p["act_bwd"]
        # what a block must keep for its backward: at least its input, the two normalised inputs, q/k/v, the
        # attention output, the MLP's pre- and post-activation (element type)
        assert prof[1]["act_bwd"] >= T * E * (d + 2 * d + 3 * d + d + 2 * f) and prof[0]["act_bwd"] == 0
        assert prof[-1]["act_bwd"] >= T * d * E + min(T, 512) * V * 4
        assert res >= cfg["M"] * T * d * E        # the boundary activations of the whole minibatch stay in HBM


def test_profile_takes_measured_times_where_the_budget_brings_them():
    """Section 4.2: the profile is measured per microbatch size.  A measurement for the forward size replaces the
    forward times, one for the backward size the backward times; other sizes fall back to flops over the rate."""
    cfg = tiny_cfg(n_blocks=2, d_model=64, n_heads=2, M=4, b=2)
    spec = B.make_spec(cfg)
    analytic, _ = B.hmy_profile(spec, 4, 2)
    meas = [dict(micro_batch=2, embed_fwd_ns=11, embed_bwd_ns=13, block_fwd_ns=1000, block_bwd_ns=3100, head_ns=700),
            dict(micro_batch=4, embed_fwd_ns=21, embed_bwd_ns=23, block_fwd_ns=1900, block_bwd_ns=6000, head_ns=1300)]
    got, _ = B.hmy_profile(spec, 4, 2, budget=B.make_budget(0, measured=meas))
    assert [(p["ns_fwd"], p["ns_bwd"]) for p in got] == [(11, 24), (1000, 3100), (1000, 3100), (700, 700)]
    assert all(p["ns_fwd_beside"] == p["ns_fwd"] and p["ns_bwd_beside"] == p["ns_bwd"] for p in got)   # none measured
    assert all(p["ns_fwd_beside"] == p["ns_fwd"] and p["ns_bwd_beside"] == p["ns_bwd"] for p in analytic)
    # times beside link traffic, where measured (never below the time alone)
    both = [dict(meas[0], embed_bwd_beside_ns=20, block_fwd_beside_ns=900, block_bwd_beside_ns=4000, head_beside_ns=800)]
    got, _ = B.hmy_profile(spec, 4, 2, budget=B.make_budget(0, measured=both))
    assert [(p["ns_fwd_beside"], p["ns_bwd_beside"]) for p in got] == [(11, 11 + 20), (1000, 4000), (1000, 4000), (800, 800)]
    got, _ = B.hmy_profile(spec, 4, 2, sched=B.make_schedule([], [], fwd_micro_batch=4), budget=B.make_budget(0, measured=meas))
    assert [(p["ns_fwd"], p["ns_bwd"]) for p in got] == [(21, 24), (1900, 3100), (1900, 3100), (1300, 700)]
    got, _ = B.hmy_profile(spec, 4, 2, sched=B.make_schedule([], [], fwd_micro_batch=8, bwd_micro_batch=1),
                           budget=B.make_budget(0, measured=meas))
    assert [p["ns_bwd"] for p in got] == [-(-p["ns_bwd"] // 2) for p in analytic] or \
        all(abs(2 * g["ns_bwd"] - a["ns_bwd"]) <= 2 for g, a in zip(got, analytic))
    assert all(g["flops_fwd"] == 4 * a["flops_fwd"] for g, a in zip(got, analytic))
    # the estimate follows: the measured schedule's time is made of the measured numbers
    sched = B.make_schedule([1, 3], [1, 3, 4])
    fast = 4_000_000_000
    ns = B.hmy_estimate(spec, sched, 4, 2, link_MBps=fast, measured=meas)
    assert abs(ns - 4 * (11 + 2 * 1000 + 700 + 2 * 3100 + 24)) <= 20


def one_layer_budget(cfg, slots=3):
    """'HBM budget sized for one layer resident': the pack-independent reserve + the largest single layer's
    backward footprint, both as the library states them."""
    prof, res = B.hmy_profile(B.make_spec(cfg), cfg["M"], cfg["b"], sched=B.make_schedule([], [], slots=slots))
    return res + max(p["mem_bwd"] for p in prof) + 512


def algorithm2_on_the_librarys_profile(cfg, budget, slots=3):
    """The oracle's Algorithm 2 (Section 4.3.1) fed with the library's own per-layer lists and with the library's
    arena size as the whole-packing test: backward packs first, then forward packs over the layers before the last
    backward pack, whose weights must fit the slots the backward packing sized."""
    spec = B.make_spec(cfg)
    like = B.make_schedule([], [], slots=slots)
    prof, res = B.hmy_profile(spec, cfg["M"], cfg["b"], sched=like)
    if budget <= res:
        return None
    R = len(prof)

    def arena_of_backward_packs(packs):
        # forward packs of one layer each: a layer's weights never need more room than the backward pack holding it
        return B.hmy_arena(spec, B.make_schedule(list(range(1, packs[-1][0] + 1)), [e for _, e in packs], slots=slots),
                           cfg["M"], cfg["b"])

    def fits(packs):
        return arena_of_backward_packs(packs)["total"] <= budget
    P_B = opk.balanced_time_packing([p["ns_bwd"] for p in prof], [p["mem_bwd"] for p in prof], budget - res, also_fits=fits)
    if P_B is None:
        return None
    RF = opk.forward_layers_given_backward(P_B)
    slot = arena_of_backward_packs(P_B)["slot_bytes"]
    P_F = opk.balanced_time_packing([p["ns_fwd"] for p in prof[:RF]], [p["mem_fwd"] for p in prof[:RF]], slots * slot)
    assert P_F is not None and R == len(prof)
    return P_F, P_B


@pytest.mark.parametrize("name", list(synth.CONFIGS))
def test_planner_is_algorithm_2_on_its_own_profile(name):
    cfg = dict(synth.CONFIGS[name])
    if cfg["budget"] is None:
        cfg["budget"] = one_layer_budget(cfg)
    spec = B.make_spec(cfg)
    s = B.hmy_plan(spec, cfg["budget"], cfg["M"], cfg["b"])
    assert (s.weight_slots, s.prefetch_distance, s.fwd_micro_batch, s.bwd_micro_batch) == (3, 1, cfg["b"], cfg["b"])
    P_F, P_B = B.schedule_packs(s)
    assert (P_F, P_B) == algorithm2_on_the_librarys_profile(cfg, cfg["budget"])
    assert B.hmy_arena(spec, s, cfg["M"], cfg["b"])["total"] <= cfg["budget"]
    # structure the paper states: forward packs cover the layers before the last
    # backward pack and are at least as large as backward packs
    assert (P_F[-1][1] if P_F else 0) == P_B[-1][0]
    if P_F and len(P_B) > 1:
        assert max(e - a_ for a_, e in P_F) >= max(e - a_ for a_, e in P_B[:-1])
    for slots in (2, 4):
        budget = max(cfg["budget"], one_layer_budget(cfg, slots))
        s2 = B.hmy_plan(spec, budget, cfg["M"], cfg["b"], slots=(slots, slots))
        assert s2.weight_slots == slots
        assert B.schedule_packs(s2) == algorithm2_on_the_librarys_profile(cfg, budget, slots)
    # fewer slots leave room for larger packs: never more of them
    assert len(B.schedule_packs(B.hmy_plan(spec, cfg["budget"], cfg["M"], cfg["b"], slots=(2, 2)))[1]) <= len(P_B)


# -------------------------------------------------------------------- arena ---

def _needs(cfg, sched_info):
    """Lower bounds on the named buffers, from what each has to hold (not from how the library lays them out)."""
    d, f, H, s_, E = cfg["d_model"], cfg["d_ffn"], cfg["n_heads"], cfg["seq_len"], _elem(cfg)
    D = cfg["M"] * cfg["b"]
    TF, TB = sched_info["fwd_micro_batch"] * s_, sched_info["bwd_micro_batch"] * s_
    return {"X": D * s_ * d * E,                 # boundary activations of the whole minibatch
            "inring": 2 * TB * d * E,            # at least double-buffered checkpoints coming in
            "outring": 2 * TF * d * E,           # and going out
            "gbig": TB * max(f, 3 * d) * E,      # gradient of the MLP's hidden layer / of q, k, v
            "gsmall": TB * d * E,
            "delta": TB * H * 4,
            "ids": D * s_ * 4, "targets": D * s_ * 4,
            "misc": 8,                           # the fp64 loss accumulator
            "kring": 2 * (3 if E == 2 else 2) * 4 * 1}


def check_arena(cfg, sched):
    spec, ospec = B.make_spec(cfg), oracle_spec(cfg)
    a = B.hmy_arena(spec, sched, cfg["M"], cfg["b"])
    regs = B.hmy_arena_regions(spec, sched, cfg["M"], cfg["b"])
    names = [n for n, _, _ in regs]
    assert len(set(names)) == len(names)
    # disjoint, aligned, inside the arena, in address order
    pos = 0
    for n, off, nbytes in regs:
        assert off % 256 == 0 and off >= pos, n
        pos = off + nbytes
    assert pos <= a["total"]
    by = {n: (off, nbytes) for n, off, nbytes in regs}
    for n, need in _needs(cfg, a).items():
        assert by[n][1] >= need, n
    assert by["kring"][1] >= 2 * (3 if _elem(cfg) == 2 else 2) * 4 * a["k_chunk_params"]
    # the slots: as many as the schedule says, each holding any pack of either pass
    slots = [by[f"slot{i}"] for i in range(a["weight_slots"])]
    assert f"slot{a['weight_slots']}" not in by and all(b == a["slot_bytes"] for _, b in slots)
    P_F, P_B = B.schedule_packs(sched)
    npar = lambda p: sum(om.layer_param_count(ospec, l) for l in range(*p))
    E = _elem(cfg)
    for p in P_F:
        assert E * npar(p) <= a["slot_bytes"]
    for p in P_B:
        assert (E + 4) * npar(p) <= a["slot_bytes"]
    # the workspace holds the largest backward pack's activations as the profile states them
    prof, res = B.hmy_profile(spec, cfg["M"], cfg["b"], sched=sched)
    assert by["acts"][1] == a["act_bytes"] >= max(sum(prof[l]["act_bwd"] for l in range(*p)) for p in P_B)
    assert res == a["reserved"] == min(off for n, off, _ in regs if n.startswith("slot"))
    return a


@pytest.mark.parametrize("name", list(synth.CONFIGS))
def test_arena_regions_are_disjoint_aligned_and_large_enough(name):
    cfg = dict(synth.CONFIGS[name])
    if cfg["budget"] is None:
        cfg["budget"] = one_layer_budget(cfg)
    spec = B.make_spec(cfg)
    for kw in (dict(), dict(search=4, slots=(2, 3)), dict(slots=(2, 2))):
        s = B.hmy_plan(spec, cfg["budget"], cfg["M"], cfg["b"], **kw)
        assert check_arena(cfg, s)["total"] <= cfg["budget"]
    # another microbatch size in each pass
    D = cfg["M"] * cfg["b"]
    s = B.hmy_plan(spec, cfg["budget"], cfg["M"], cfg["b"])
    for uF, uB in ((D, cfg["b"]), (1, cfg["b"]), (cfg["b"], 1)):
        s.fwd_micro_batch, s.bwd_micro_batch = uF, uB
        a = check_arena(cfg, s)
        assert (a["fwd_micro_batch"], a["bwd_micro_batch"]) == (uF, uB)


def test_arena_regions_on_random_small_models():
    rng = np.random.default_rng(3)
    for _ in range(40):
        H = int(rng.choice([1, 2, 4]))
        cfg = tiny_cfg(n_blocks=int(rng.integers(1, 6)), d_model=H * 32, n_heads=H, d_ffn=int(rng.choice([64, 136])),
                       seq_len=int(rng.choice([8, 24])), vocab=int(rng.integers(17, 900)),
                       precision=str(rng.choice(["fp32", "bf16"])), M=int(rng.integers(1, 5)), b=int(rng.choice([1, 2, 4])))
        R = cfg["n_blocks"] + 2
        packs = list(all_packings(R))
        P_B = packs[int(rng.integers(len(packs)))]
        fw = list(all_packings(P_B[-1][0])) if P_B[-1][0] else [[]]
        P_F = fw[int(rng.integers(len(fw)))]
        slots = int(rng.integers(2, 5))
        D = cfg["M"] * cfg["b"]
        divs = [u for u in range(1, D + 1) if D % u == 0]
        sched = B.make_schedule([e for _, e in P_F], [e for _, e in P_B], slots=slots, distance=int(rng.integers(1, slots)),
                                fwd_micro_batch=int(rng.choice(divs)), bwd_micro_batch=int(rng.choice(divs)))
        check_arena(cfg, sched)


# ---------------------------------------------------------------- estimate ---

def simulate_like_the_library(cfg, sched, link_MBps=40000, compute_GFLOPs=420000, measured=None):
    """The oracle's event-driven simulation (oracle/simulate.py) of the schedule, fed with the library's per-layer
    times (hmy_profile) and exact byte times.  Returns (ns as a Fraction, number of operations)."""
    from fractions import Fraction as Fr
    from oracle import simulate as osim
    spec, ospec = B.make_spec(cfg), oracle_spec(cfg)
    a = B.hmy_arena(spec, sched, cfg["M"], cfg["b"])
    prof, _ = B.hmy_profile(spec, cfg["M"], cfg["b"], sched=sched,
                            budget=B.make_budget(0, link_MBps=link_MBps, compute_GFLOPs=compute_GFLOPs, measured=measured))
    P_F, P_B = B.schedule_packs(sched)
    w_c, k_B, g_B = osw.bytes_per_param(cfg["precision"])
    D = cfg["M"] * cfg["b"]
    uF, uB = a["fwd_micro_batch"], a["bwd_micro_batch"]
    row = cfg["seq_len"] * cfg["d_model"] * w_c
    per_byte = Fr(1000, link_MBps)
    ops = osim.iteration_ops(ospec, P_F, P_B, [p["ns_fwd"] for p in prof], [p["ns_bwd"] for p in prof], D // uF, D // uB,
                             uF * row, uB * row, w_c, k_B, g_B, per_byte, per_byte, slots=a["weight_slots"],
                             distance=a["prefetch_distance"], update_on_host=bool(sched.update_site),
                             export_gradients=not sched.gradients,
                             t_fwd_beside=[p["ns_fwd_beside"] for p in prof], t_bwd_beside=[p["ns_bwd_beside"] for p in prof])
    return max(e for _, e in osim.run(ops).values()), len(ops)


def assert_estimate_matches_simulation(cfg, sched, **rates):
    want, n_ops = simulate_like_the_library(cfg, sched, **rates)
    got = B.hmy_estimate(B.make_spec(cfg), sched, cfg["M"], cfg["b"], **rates)
    # the library rounds every operation's time up to a whole nanosecond (the CPU's down); the simulation is exact
    assert abs(got - want) <= n_ops + 1, (got, float(want), B.schedule_packs(sched))
    return got


def test_estimate_on_schedules_worked_by_hand():
    """Literal expectations.  Model: one block, d = 32, one head, f = 32, s = 8, V = 16, fp32, one sequence per
    microbatch.  Parameters: embedding 16*32 + 8*32 = 768, block 4*32^2 + 2*32*32 + 9*32 + 32 = 6464, head
    2*32 + 16*32 = 576.  Forward flops per microbatch (T = 8 tokens): embedding T d = 256, block
    T (8 d^2 + 4 d f + 2 s d) = 8 * 12800 = 102400, head 2 T d V = 8192.  Rates: 1 GFLOP/s = 1 flop per ns,
    1000 MB/s = 1 byte per ns; so W = 4 B/param, K = 8 B/param, update out = 16 B/param (gradient exported) in ns,
    backward tasks three times the forward flops, a checkpoint 8*32*4 = 1024 ns per microbatch.

    (a) P_F = [0,2), P_B = [0,2) [2,3), two microbatches, three slots:
        W0 = 4*7232 = 28928, C0 = 2*102656 = 205312; W1 = 2304, C1 = 2*24576 = 49152, K1 = 4608, Out1 = 9216;
        W2 = 28928, C2 = 2*307968 = 615936, K2 = 57856, Out2 = 115712.
        W0 0-28928; C0 -234240; W1 (asked at 28928) -31232; C1 234240-283392; W2 (asked at 234240) -263168;
        K1 283392-288000; Out1 283392-292608; C2 283392-899328; K2 899328-957184; Out2 899328-1015040.
    (b) the same with the update on the host (CPU at 6 parameters per ns): Out1 = 4*576 = 2304, Cpu1 = 96,
        Out2 = 4*7232 = 28928, Cpu2 = 7232 // 6 = 1205: C2 ends 899328, Out2 -928256, Cpu2 -929461.
    (c) one layer per pack, P_F = [0,1) [1,2), P_B = [0,1) [1,2) [2,3), one microbatch, TWO slots, link at
        100 MB/s (10 ns per byte): W 30720 / 258560 / 23040; C 256 / 102400 forward, 24576 / 307200 / 768 backward;
        K 46080 / 517120 / 61440, Out 92160 / 1034240 / 122880; the block's checkpoint 10240 each way.
        W0 0-30720; C0 -30976; W1 (asked at 30720) -289280; Sout1 (asked when C1 starts, 289280) -299520;
        C1 289280-391680; W2 = head (asked at 289280; slot of visit 0, free at 30976) -312320; C2 391680-416256;
        W3 = block (asked at 391680; slot of visit 1, free at 391680) 391680-650240; K2 (asked at 416256) 650240-711680;
        Out2 416256-539136, held to 711680 by K2; Sin3 (asked when C3 starts) ...; C3 650240-957440;
        Sin3 711680-721920; W4 (asked at 650240; slot of visit 2, free at 711680) 721920-752640; K3 957440-1474560;
        Out3 957440-1991680; C4 957440-958208; K4 1474560-1536000; Out4 1991680-2114560.
    (d) as (c) with three slots: W3 does not wait for a slot either way here (391680 is when it is asked for), and
        W4 needs visit 1's slot, long free: same times, 2114560."""
    cfg = tiny_cfg(n_blocks=1, d_model=32, n_heads=1, d_ffn=32, seq_len=8, vocab=16, precision="fp32", M=2, b=1)
    spec = B.make_spec(cfg)
    prof, _ = B.hmy_profile(spec, 2, 1, budget=B.make_budget(0, compute_GFLOPs=1))
    assert [(p["params"], p["ns_fwd"], p["ns_bwd"]) for p in prof] == [(768, 256, 768), (6464, 102400, 307200),
                                                                       (576, 8192, 24576)]
    rates = dict(link_MBps=1000, compute_GFLOPs=1)
    a = B.make_schedule([2], [2, 3])
    assert B.hmy_estimate(spec, a, 2, 1, **rates) == 1015040
    a.update_site = B.HMY_UPDATE_ON_HOST
    assert B.hmy_estimate(spec, a, 2, 1, **rates) == 929461
    # (e) schedule (a) with per-layer times given as measurements (microbatch size 1: embedding 256 forward, 256
    #     backward, so 512 in a backward task; block 102400 / 307200; head 8192) and the block's backward time beside
    #     link traffic twice its time alone (614400):
    #     W0 0-28928; C0 = 2*(256+102400) -234240; W1 -31232; C1 = 2*8192 starts at 234240 with nothing outgoing
    #     queued: as alone -> 250624; W2 (asked at 234240) -263168; K1 (asked at 250624, behind W2) 263168-267776;
    #     Out1 250624-259840, held to 267776 by K1; C2 = 2*(512+307200) = 615424 alone, 1229824 beside traffic,
    #     starts at 263168 (its weights) while the outgoing link is busy until 267776: a backlog of 4608 ns, so it
    #     takes 615424 + 614400 * 4608 / 615424 = 620024 (rounded down) -> 883192; K2 -941048; Out2 883192-998904.
    meas = [dict(micro_batch=1, embed_fwd_ns=256, embed_bwd_ns=256, block_fwd_ns=102400, block_bwd_ns=307200, head_ns=8192,
                 block_bwd_beside_ns=614400)]
    e = B.make_schedule([2], [2, 3])
    assert B.hmy_estimate(spec, e, 2, 1, link_MBps=1000, measured=meas) == 998904
    assert B.hmy_estimate(spec, e, 2, 1, link_MBps=1000, measured=[dict(meas[0], block_bwd_beside_ns=0)]) == 994304
    slow = dict(link_MBps=100, compute_GFLOPs=1)
    stretched = B.hmy_estimate(spec, e, 2, 1, link_MBps=100, measured=meas)
    assert stretched > B.hmy_estimate(spec, e, 2, 1, link_MBps=100, measured=[dict(meas[0], block_bwd_beside_ns=0)])
    assert_estimate_matches_simulation(cfg, e, link_MBps=100, measured=meas)
    c = B.make_schedule([1, 2], [1, 2, 3], slots=2)
    assert B.hmy_estimate(spec, c, 1, 1, **slow) == 2114560
    c.weight_slots = 3
    assert B.hmy_estimate(spec, c, 1, 1, **slow) == 2114560
    # and the oracle's simulation says the same of all four
    cfg1 = dict(cfg, M=1)
    for cfg_, sched, r in ((cfg, B.make_schedule([2], [2, 3]), rates), (cfg, a, rates), (cfg1, c, slow)):
        assert_estimate_matches_simulation(cfg_, sched, **r)


@pytest.mark.parametrize("name", ["gpt2m", "gpt2xl", "bertl", "gpt6b7"])
def test_estimate_equals_the_oracles_simulation_on_the_workloads(name):
    cfg = synth.CONFIGS[name]
    spec = B.make_spec(cfg)
    D = cfg["M"] * cfg["b"]
    for kw in (dict(), dict(search=4, slots=(2, 4)), dict(search=4, update_site=B.HMY_UPDATE_ON_HOST)):
        s = B.hmy_plan(spec, cfg["budget"], cfg["M"], cfg["b"], **kw)
        for rates in (dict(), dict(link_MBps=25000, compute_GFLOPs=600000)):
            assert_estimate_matches_simulation(cfg, s, **rates)
        for slots, dist in ((2, 1), (3, 2), (4, 3)):
            s.weight_slots, s.prefetch_distance = slots, dist
            assert_estimate_matches_simulation(cfg, s)
        s.weight_slots, s.prefetch_distance = 3, 1
        s.gradients = B.HMY_GRADIENTS_ON_DEVICE
        assert_estimate_matches_simulation(cfg, s)
        s.gradients = B.HMY_GRADIENTS_EXPORTED
        s.fwd_micro_batch, s.bwd_micro_batch = (D if D <= 64 else cfg["b"] * 2), cfg["b"]
        assert_estimate_matches_simulation(cfg, s)


def test_estimate_equals_the_oracles_simulation_on_every_packing_of_a_small_model():
    cfg = tiny_cfg(n_blocks=3, d_model=64, n_heads=2, d_ffn=128, seq_len=16, vocab=50, precision="bf16", M=4, b=2)
    rng = np.random.default_rng(11)
    n = 0
    meas = [dict(micro_batch=2, embed_fwd_ns=300, embed_bwd_ns=900, block_fwd_ns=9000, block_bwd_ns=31000, head_ns=5000,
                 embed_bwd_beside_ns=1300, block_fwd_beside_ns=9500, block_bwd_beside_ns=40000, head_beside_ns=5900),
            dict(micro_batch=8, embed_fwd_ns=1000, embed_bwd_ns=3000, block_fwd_ns=30000, block_bwd_ns=99000, head_ns=17000,
                 block_bwd_beside_ns=120000)]
    for P_B in all_packings(5):
        fw = list(all_packings(P_B[-1][0])) if P_B[-1][0] else [[]]
        for P_F in fw[::2]:
            slots = int(rng.integers(2, 5))
            sched = B.make_schedule([e for _, e in P_F], [e for _, e in P_B], slots=slots, distance=int(rng.integers(1, slots)),
                                    update_site=int(rng.integers(0, 2)), gradients=int(rng.integers(0, 2)),
                                    fwd_micro_batch=int(rng.choice([1, 2, 4, 8])), bwd_micro_batch=int(rng.choice([1, 2, 8])))
            link = int(rng.choice([50, 2000, 40000]))
            assert_estimate_matches_simulation(cfg, sched, link_MBps=link, compute_GFLOPs=int(rng.choice([1, 30, 5000])))
            assert_estimate_matches_simulation(cfg, sched, link_MBps=link, measured=meas)
            n += 1
    assert n > 25


@pytest.mark.parametrize("name", ["gpt2m", "gpt2xl", "bertl", "gpt6b7"])
def test_configuration_search_keeps_the_smallest_estimate_of_its_candidates(name):
    """Algorithm 1's selection rule: the searched configuration is valid, fits the budget, and no candidate that
    the test can name itself -- Algorithm 2's packing for any slot count, with any prefetch distance -- has a smaller
    estimate under the same rates; sweeping more never returns a longer estimate."""
    cfg = synth.CONFIGS[name]
    spec = B.make_spec(cfg)
    for rates in (dict(), dict(link_MBps=25000, compute_GFLOPs=600000)):
        for site in (B.HMY_UPDATE_ON_DEVICE, B.HMY_UPDATE_ON_HOST):
            best = B.hmy_plan(spec, cfg["budget"], cfg["M"], cfg["b"], search=8, slots=(2, 4), update_site=site, **rates)
            assert best.update_site == site
            ns = B.hmy_estimate(spec, best, cfg["M"], cfg["b"], **rates)
            assert check_arena(cfg, best)["total"] <= cfg["budget"]
            narrower = B.hmy_plan(spec, cfg["budget"], cfg["M"], cfg["b"], search=2, update_site=site, **rates)
            assert ns <= B.hmy_estimate(spec, narrower, cfg["M"], cfg["b"], **rates)
            for slots in (2, 3, 4):
                got = algorithm2_on_the_librarys_profile(cfg, cfg["budget"], slots)
                for dist in range(1, slots):
                    cand = B.make_schedule([e for _, e in got[0]], [e for _, e in got[1]], slots=slots, distance=dist,
                                           update_site=site)
                    assert ns <= B.hmy_estimate(spec, cand, cfg["M"], cfg["b"], **rates)
            # less traffic, never a longer estimate
            if site == B.HMY_UPDATE_ON_HOST:
                dev = B.hmy_plan(spec, cfg["budget"], cfg["M"], cfg["b"], search=8, slots=(2, 4), **rates)
                assert ns <= B.hmy_estimate(spec, dev, cfg["M"], cfg["b"], **rates)


def test_configuration_search_over_microbatch_sizes():
    """Algorithm 1 sweeps U_B, then U_F (the divisors of the minibatch up to the caps).  With the analytic profile a
    microbatch size changes no task's time, only the bytes it keeps: the sweep can only find packings that the
    caller's size could not fit, and it must return the caller's size when nothing beats it.  With measured profiles
    that make one size faster per sequence the sweep must pick that size."""
    cfg = dict(synth.CONFIGS["bertl"])
    spec = B.make_spec(cfg)
    base = B.hmy_plan(spec, cfg["budget"], cfg["M"], cfg["b"], search=2)
    swept = B.hmy_plan(spec, cfg["budget"], cfg["M"], cfg["b"], search=2, max_fwd_micro_batch=32, max_bwd_micro_batch=16)
    ns_base, ns_swept = (B.hmy_estimate(spec, s, cfg["M"], cfg["b"]) for s in (base, swept))
    assert ns_swept <= ns_base and check_arena(cfg, swept)["total"] <= cfg["budget"]
    assert 256 % swept.fwd_micro_batch == 0 and 256 % swept.bwd_micro_batch == 0
    assert swept.fwd_micro_batch <= 32 and swept.bwd_micro_batch <= 16
    # measured: 16 sequences at a time run the forward pass at 0.7 of the time per sequence of 8, backward sizes equal
    t = lambda u, k: dict(micro_batch=u, embed_fwd_ns=1000 * u, embed_bwd_ns=2000 * u, block_fwd_ns=int(k * 300000 * u),
                          block_bwd_ns=1000000 * u, head_ns=800000 * u)
    sizes = (1, 2, 4, 8, 16, 32)              # every size the sweep may visit (a size without a measurement falls
    meas = [t(u, 0.7 if u == 16 else 1.0) for u in sizes]                    # back to flops over the rate)
    pick = B.hmy_plan(spec, cfg["budget"], cfg["M"], cfg["b"], max_fwd_micro_batch=32, measured=meas)
    assert pick.fwd_micro_batch == 16 and pick.bwd_micro_batch == 8
    keep = B.hmy_plan(spec, cfg["budget"], cfg["M"], cfg["b"], max_fwd_micro_batch=32, measured=[t(u, 1.0) for u in sizes])
    assert keep.fwd_micro_batch == 8          # ties go to the caller's own size


def test_runtime_estimate_closed_forms():
    """Degenerate cases of the estimator that can be worked by hand: with an
    infinitely fast link the estimate is the sum of the visits' compute times; with
    infinitely fast compute it is the serial swap time of the dominant direction."""
    cfg = tiny_cfg(n_blocks=3, d_model=64, n_heads=2, d_ffn=128, seq_len=16, vocab=50, precision="bf16", M=2, b=2)
    spec = B.make_spec(cfg)
    sched = B.make_schedule([2, 4], [2, 4, 5])
    rate = 1000                                      # GFLOP/s = flops per ns
    prof, _ = B.hmy_profile(spec, 2, 2, budget=B.make_budget(0, compute_GFLOPs=rate))
    per_visit = [2 * sum(prof[l]["ns_fwd"] for l in r) for r in (range(0, 2), range(2, 4))] + \
                [2 * sum(prof[l]["ns_bwd"] for l in r) for r in (range(4, 5), range(2, 4), range(0, 2))]
    fast_link = B.hmy_estimate(spec, sched, 2, 2, link_MBps=4_000_000_000, compute_GFLOPs=rate)
    assert abs(fast_link - sum(per_visit)) <= 12     # + a few ns of (rounded-up) transfers
    n = sum(p["params"] for p in prof)
    slow = B.hmy_estimate(spec, sched, 2, 2, link_MBps=1, compute_GFLOPs=4_000_000_000)
    # device->host moves (12 + 2 + 4) B/param once; host->device moves 12 B/param of state + weights twice minus the last pack
    d2h_ns = 18 * n * 1000
    ck = 2 * 2 * 16 * 64 * 2 * 1000                  # one checkpoint (the pack starting at layer 2) each way
    assert d2h_ns <= slow <= d2h_ns + ck + 2 * 2 * n * 1000 + 12 * n * 1000 + ck + 100
    # the update on the host: only the weights come in and only the 4 B/param gradient goes out; with a slow link
    # the weight loads (twice, minus the last pack) are the longer queue, the CPU (6 parameters/ns) comes after
    host = B.make_schedule([2, 4], [2, 4, 5], update_site=B.HMY_UPDATE_ON_HOST)
    slow_h = B.hmy_estimate(spec, host, 2, 2, link_MBps=1, compute_GFLOPs=4_000_000_000)
    n_last = prof[4]["params"]
    w_in_ns = 2 * (2 * n - n_last) * 1000
    assert w_in_ns <= slow_h <= w_in_ns + 2 * ck + 4 * n * 1000 + n // 6 + 100
    fast_h = B.hmy_estimate(spec, host, 2, 2, link_MBps=4_000_000_000, compute_GFLOPs=rate)
    first_pack = prof[0]["params"] + prof[1]["params"]        # updated last: nothing left to hide its CPU time
    assert abs(fast_h - (fast_link + first_pack // 6)) <= 12


def test_tiny_config_budget_gives_one_layer_per_pack():
    cfg = dict(synth.CONFIGS["tiny"])
    spec = B.make_spec(cfg)
    s = B.hmy_plan(spec, one_layer_budget(cfg), cfg["M"], cfg["b"])
    P_F, P_B = B.schedule_packs(s)
    assert P_B == [(i, i + 1) for i in range(6)]
    # a forward slot only holds weights (no fp32 gradients), so in fp32 up to two
    # layers share it: forward packs are at least as large as backward packs
    assert P_F[0][0] == 0 and P_F[-1][1] == 5 and all(1 <= e - a <= 2 for a, e in P_F)
    # the explicit one-layer-per-pack schedule is valid under the same budget
    a = B.hmy_arena(spec, B.make_schedule([1, 2, 3, 4, 5], [1, 2, 3, 4, 5, 6]), cfg["M"], cfg["b"])
    assert a["total"] <= one_layer_budget(cfg)


def test_planner_is_algorithm_2_on_random_small_models_and_budgets():
    rng = np.random.default_rng(0)
    n_checked = 0
    for _ in range(60):
        H = int(rng.choice([1, 2, 4]))
        dh = int(rng.choice([32, 64]))
        cfg = tiny_cfg(n_blocks=int(rng.integers(1, 9)), d_model=H * dh, n_heads=H,
                       d_ffn=int(rng.choice([64, 128, 512])), seq_len=int(rng.choice([8, 16, 64])),
                       vocab=int(rng.integers(17, 3000)), causal=int(rng.integers(0, 2)),
                       precision=str(rng.choice(["fp32", "bf16"])), M=int(rng.integers(1, 5)), b=int(rng.integers(1, 4)))
        spec = B.make_spec(cfg)
        slots = int(rng.integers(2, 5))
        lo = one_layer_budget(cfg, slots)
        prof, _ = B.hmy_profile(spec, cfg["M"], cfg["b"], sched=B.make_schedule([], [], slots=slots))
        hi = lo + sum(p["mem_bwd"] for p in prof)
        for budget in (lo // 2, lo, (lo + hi) // 2, int(lo + 0.3 * (hi - lo)), hi + 10 ** 6):
            want = algorithm2_on_the_librarys_profile(cfg, budget, slots)
            try:
                got = B.schedule_packs(B.hmy_plan(spec, budget, cfg["M"], cfg["b"], slots=(slots, slots)))
            except B.HmyError as e:
                assert e.code == B.HMY_E_BUDGET_TOO_SMALL and want is None
                continue
            assert want is not None and got == (want[0], want[1]), (cfg, budget)
            n_checked += 1
    assert n_checked > 100


# ---------------------------------------------------------------- counters ---

def _cmp_counters(cfg, P_F, P_B):
    spec, ospec = B.make_spec(cfg), oracle_spec(cfg)
    sched = B.make_schedule([e for _, e in P_F], [e for _, e in P_B])
    got = B.hmy_count_swaps(spec, sched, cfg["M"], cfg["b"])
    want = osw.closed_form(ospec, P_F, P_B, cfg["M"], cfg["b"], cfg["precision"])
    assert got["h2d"] == want["h2d"] and got["d2h"] == want["d2h"]
    assert want == osw.ledger(ospec, P_F, P_B, cfg["M"], cfg["b"], cfg["precision"])
    # the comparison order over the same packs
    sched.order = B.HMY_ORDER_MICROBATCH_MAJOR
    got_mm = B.hmy_count_swaps(spec, sched, cfg["M"], cfg["b"])
    want_mm = osw.closed_form_microbatch_major(ospec, P_F, P_B, cfg["M"], cfg["b"], cfg["precision"])
    assert got_mm["h2d"] == want_mm["h2d"] and got_mm["d2h"] == want_mm["d2h"]
    # the update task on the CPU, in both orders
    for order, cf in ((B.HMY_ORDER_LAYER_PACK_MAJOR, osw.closed_form),
                      (B.HMY_ORDER_MICROBATCH_MAJOR, osw.closed_form_microbatch_major)):
        sched.order, sched.update_site = order, B.HMY_UPDATE_ON_HOST
        got_h = B.hmy_count_swaps(spec, sched, cfg["M"], cfg["b"])
        want_h = cf(ospec, P_F, P_B, cfg["M"], cfg["b"], cfg["precision"], update_on_host=True)
        assert got_h["h2d"] == want_h["h2d"] and got_h["d2h"] == want_h["d2h"]
        # the consumed gradient dropped on the device instead of exported, at both update sites
        for site in (B.HMY_UPDATE_ON_DEVICE, B.HMY_UPDATE_ON_HOST):
            sched.update_site, sched.gradients = site, B.HMY_GRADIENTS_ON_DEVICE
            got_d = B.hmy_count_swaps(spec, sched, cfg["M"], cfg["b"])
            want_d = cf(ospec, P_F, P_B, cfg["M"], cfg["b"], cfg["precision"], update_on_host=bool(site),
                        export_gradients=False)
            assert got_d["h2d"] == want_d["h2d"] and got_d["d2h"] == want_d["d2h"]
        sched.gradients = B.HMY_GRADIENTS_EXPORTED
    # slots, prefetch distance and the swap-out mechanism change when bytes move, never how many; another microbatch
    # size in either pass cuts the same checkpoints differently (closed form and ledger with M_F, b_F)
    D = cfg["M"] * cfg["b"]
    for kw in (dict(slots=2), dict(slots=4, distance=3), dict(swap_out=B.HMY_SWAP_OUT_MEMCPY),
               dict(fwd_micro_batch=D), dict(fwd_micro_batch=1, slots=2), dict(bwd_micro_batch=1, fwd_micro_batch=cfg["b"])):
        for site in (B.HMY_UPDATE_ON_DEVICE, B.HMY_UPDATE_ON_HOST):
            alt = B.make_schedule([e for _, e in P_F], [e for _, e in P_B], update_site=site, **kw)
            got_a = B.hmy_count_swaps(spec, alt, cfg["M"], cfg["b"])
            uF, uB = kw.get("fwd_micro_batch", cfg["b"]), kw.get("bwd_micro_batch", cfg["b"])
            for f in (osw.closed_form, osw.ledger):
                want_a = f(ospec, P_F, P_B, D // uB, uB, cfg["precision"], update_on_host=bool(site), M_F=D // uF, b_F=uF)
                assert got_a["h2d"] == want_a["h2d"] and got_a["d2h"] == want_a["d2h"], kw
            if uB == cfg["b"]:
                ref = dict(got) if site == B.HMY_UPDATE_ON_DEVICE else None
                if ref:
                    assert got_a["h2d"] == got["h2d"] and got_a["d2h"] == got["d2h"]
    return got


@pytest.mark.parametrize("name", list(synth.CONFIGS))
def test_swap_counters_equal_closed_form_on_planned_configs(name):
    cfg = dict(synth.CONFIGS[name])
    if cfg["budget"] is None:
        cfg["budget"] = one_layer_budget(cfg)
    P_F, P_B = B.schedule_packs(B.hmy_plan(B.make_spec(cfg), cfg["budget"], cfg["M"], cfg["b"]))
    got = _cmp_counters(cfg, P_F, P_B)
    # the headline of the method: weights come in once per pass, not once per microbatch
    E = 2 if cfg["precision"] == "bf16" else 4
    n = B.hmy_model_size(B.make_spec(cfg))[1]
    assert got["h2d"]["W"] < 2 * E * n
    assert got["d2h"]["W"] == E * n and got["h2d"]["dW"] == 0 and got["h2d"]["XY"] == got["d2h"]["XY"] == 0
    # ... and what the comparison order pays instead (Section 3: M times the weights; appendix: gradients M-1 / M times)
    sched = B.make_schedule([e for _, e in P_F], [e for _, e in P_B], order=B.HMY_ORDER_MICROBATCH_MAJOR)
    mm = B.hmy_count_swaps(B.make_spec(cfg), sched, cfg["M"], cfg["b"])
    assert mm["h2d"]["W"] == cfg["M"] * got["h2d"]["W"]
    assert mm["h2d"]["dW"] == (cfg["M"] - 1) * 4 * n and mm["d2h"]["dW"] == cfg["M"] * 4 * n


@pytest.mark.parametrize("precision", ["fp32", "bf16"])
def test_swap_counters_equal_closed_form_on_every_packing_of_a_small_model(precision):
    cfg = tiny_cfg(n_blocks=3, d_model=32, n_heads=1, d_ffn=64, seq_len=8, vocab=40, precision=precision, M=3, b=2)
    R = 5
    n = 0
    for P_B in all_packings(R):
        last_start = P_B[-1][0]
        for P_F in (list(all_packings(last_start)) if last_start else [[]]):
            _cmp_counters(cfg, P_F, P_B)
            n += 1
    assert n > 30


# ------------------------------------------------------- update on the host ---

@pytest.mark.parametrize("precision,threads,n", [("fp32", 1, 1000), ("fp32", 5, 100003), ("bf16", 3, 64 * 7 + 1),
                                                 ("bf16", 16, 300007), ("bf16", 0, 17)])
def test_host_adam_matches_the_oracle_update(precision, threads, n):
    """The CPU-side Weight Update (Section 4.4) against the oracle's Adam, element by
    element: fp32 arithmetic against fp64, so 1e-6 of the largest value; the bf16 weight
    is exactly the round-to-nearest-even of the fp32 master it was made from."""
    rng = np.random.default_rng(n)
    w = (rng.standard_normal(n) * 0.05).astype(np.float32)
    g = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    g[::7] = 0.0
    m = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    v = (rng.random(n) * 1e-5).astype(np.float32)
    f32 = lambda x: float(np.float32(x))
    hp = om.AdamHP(lr=f32(3e-4), beta1=f32(0.9), beta2=f32(0.999), eps=f32(1e-8), step=7)
    w_ref, m_ref, v_ref = om.adam_update(w.astype(np.float64), g.astype(np.float64), m.astype(np.float64),
                                         v.astype(np.float64), hp)
    mixed = precision == "bf16"
    master, mm, vv, gg = w.copy(), m.copy(), v.copy(), g.copy()
    w16 = np.zeros(n, np.uint16)
    ptr = lambda a: a.ctypes.data
    if mixed:
        B.hmy_host_adam(B.HMY_PREC_BF16, ptr(gg), ptr(master), ptr(mm), ptr(vv), ptr(w16), n, hp.lr, hp.beta1, hp.beta2,
                        hp.eps, hp.step, threads)
    else:
        B.hmy_host_adam(B.HMY_PREC_FP32, ptr(gg), None, ptr(mm), ptr(vv), ptr(master), n, hp.lr, hp.beta1, hp.beta2,
                        hp.eps, hp.step, threads)
    assert np.array_equal(gg, g)
    assert np.abs(mm - m_ref).max() < 1e-6 * np.abs(m_ref).max()
    assert np.abs(vv - v_ref).max() < 1e-6 * np.abs(v_ref).max()
    # the stored fp32 weight carries its own rounding (half an ulp of |w|) on top of the update's
    assert np.abs(master - w_ref).max() < 2.0 ** -24 * np.abs(w).max() + 1e-6 * np.abs(w_ref - w).max()
    if mixed:
        want = synth.round_bf16(master)
        got = (w16.astype(np.uint32) << 16).view(np.float32)
        assert np.array_equal(got, want)


def test_host_adam_argument_errors():
    a = np.zeros(8, np.float32)
    p = a.ctypes.data
    for args in ((B.HMY_PREC_BF16, p, None, p, p, p, 8), (B.HMY_PREC_FP32, p, p, p, p, p, 8), (7, p, None, p, p, p, 8),
                 (B.HMY_PREC_FP32, None, None, p, p, p, 8)):
        with pytest.raises(B.HmyError) as e:
            B.hmy_host_adam(*args, 1e-3, 0.9, 0.999, 1e-8, 1)
        assert e.value.code == B.HMY_E_INVALID
    with pytest.raises(B.HmyError):
        B.hmy_host_adam(B.HMY_PREC_FP32, p, None, p, p, p, 8, 1e-3, 0.9, 0.999, 1e-8, 0)    # step is 1-based


# ------------------------------------------------------------------ errors ---

def test_error_paths_return_codes_not_crashes():
    cfg = tiny_cfg(d_model=64, n_heads=2)
    spec = B.make_spec(cfg)
    with pytest.raises(B.HmyError) as e:
        B.hmy_plan(spec, 1000, 2, 2)
    assert e.value.code == B.HMY_E_BUDGET_TOO_SMALL
    bad = B.make_spec(dict(cfg, d_model=60))          # head dim 30
    with pytest.raises(B.HmyError) as e:
        B.hmy_model_size(bad)
    assert e.value.code == B.HMY_E_INVALID
    with pytest.raises(B.HmyError) as e:                # packs do not cover all layers
        B.hmy_arena(spec, B.make_schedule([], [2, 3]), 2, 2)
    assert e.value.code == B.HMY_E_BAD_SCHEDULE
    with pytest.raises(B.HmyError) as e:                # forward packs must stop before the last backward pack
        B.hmy_arena(spec, B.make_schedule([4], [2, 4]), 2, 2)
    assert e.value.code == B.HMY_E_BAD_SCHEDULE
    with pytest.raises(B.HmyError) as e:
        B.hmy_count_swaps(spec, B.make_schedule([1], [2, 4]), 2, 2)
    assert e.value.code == B.HMY_E_BAD_SCHEDULE
    with pytest.raises(B.HmyError) as e:                # a task order that does not exist
        B.hmy_count_swaps(spec, B.make_schedule([2], [2, 4], order=2), 2, 2)
    assert e.value.code == B.HMY_E_BAD_SCHEDULE
    with pytest.raises(B.HmyError) as e:                # nor this update site
        B.hmy_count_swaps(spec, B.make_schedule([2], [2, 4], update_site=-1), 2, 2)
    assert e.value.code == B.HMY_E_BAD_SCHEDULE
    with pytest.raises(B.HmyError) as e:                # nor this way to dispose of gradients
        B.hmy_count_swaps(spec, B.make_schedule([2], [2, 4], gradients=2), 2, 2)
    assert e.value.code == B.HMY_E_BAD_SCHEDULE
    with pytest.raises(B.HmyError) as e:                # nor this residency
        B.hmy_count_swaps(spec, B.make_schedule([2], [2, 4], resident_state=5), 2, 2)
    assert e.value.code == B.HMY_E_BAD_SCHEDULE
    for bad in (dict(swap_out=2), dict(slots=1), dict(slots=5), dict(slots=3, distance=3), dict(distance=-1),
                dict(fwd_micro_batch=3), dict(bwd_micro_batch=8), dict(fwd_micro_batch=1, order=B.HMY_ORDER_MICROBATCH_MAJOR)):
        with pytest.raises(B.HmyError) as e:            # slots 2..4, distance below them, sizes dividing the minibatch of 4
            B.hmy_count_swaps(spec, B.make_schedule([2], [2, 4], **bad), 2, 2)
        assert e.value.code == B.HMY_E_BAD_SCHEDULE, bad
    with pytest.raises(B.HmyError) as e:
        B.hmy_plan(spec, 1 << 30, 2, 2, slots=(4, 2))
    assert e.value.code == B.HMY_E_INVALID
    # without an engine (and a budget) there is nothing resident: the dry count is the swapped one
    assert B.hmy_count_swaps(spec, B.make_schedule([2], [2, 4], resident_state=1), 2, 2) == \
        B.hmy_count_swaps(spec, B.make_schedule([2], [2, 4]), 2, 2)
    assert B.lib.hmy_strerror(B.HMY_E_HIP) == b"HIP runtime error"
    assert B.lib.hmy_model_size(None, None, None) == B.HMY_E_INVALID


def test_bench_refuses_more_than_one_gpu_and_has_no_cpu_fallback():
    """One GPU only: `--gpus N` with N > 1 ends with a message and a non-zero status before anything is loaded;
    without a GPU the benchmark says so instead of timing something else."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and not r.stdout.strip()
    import torch
    if not torch.cuda.is_available():
        r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--steps", "1", "--warmup", "0"],
                           capture_output=True, text=True, timeout=300)
        assert r.returncode != 0 and "needs a GPU" in r.stderr and not r.stdout.strip()

