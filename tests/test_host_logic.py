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
             "hmy_stats", "hmy_tensor_desc", "hmy_layer_profile", "hmy_arena_plan", "hmy_gemm_desc"]
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


@pytest.mark.parametrize("name", list(synth.CONFIGS))
def test_profile_and_reserve_match_the_oracle_model(name):
    cfg = synth.CONFIGS[name]
    spec, ospec = B.make_spec(cfg), oracle_spec(cfg)
    prof, res = B.hmy_profile(spec, cfg["M"], cfg["b"])
    assert prof == opk.layer_profile(ospec, cfg["M"], cfg["b"], cfg["precision"])
    assert res == opk.reserved_bytes(ospec, cfg["M"], cfg["b"], cfg["precision"])


def one_layer_budget(cfg):
    """'HBM budget sized for one layer resident': reserve + the largest single
    layer's backward footprint."""
    ospec = oracle_spec(cfg)
    prof = opk.layer_profile(ospec, cfg["M"], cfg["b"], cfg["precision"])
    return opk.reserved_bytes(ospec, cfg["M"], cfg["b"], cfg["precision"]) + max(p["mem_bwd"] for p in prof) + 512


@pytest.mark.parametrize("name", list(synth.CONFIGS))
def test_planner_returns_the_oracles_packs(name):
    cfg = dict(synth.CONFIGS[name])
    if cfg["budget"] is None:
        cfg["budget"] = one_layer_budget(cfg)
    spec, ospec = B.make_spec(cfg), oracle_spec(cfg)
    s = B.hmy_plan(spec, cfg["budget"], cfg["M"], cfg["b"])
    P_F, P_B = B.schedule_packs(s)
    want = opk.plan(ospec, cfg["budget"], cfg["M"], cfg["b"], cfg["precision"])
    assert want is not None and (P_F, P_B) == (want[0], want[1])
    a = B.hmy_arena(spec, s, cfg["M"], cfg["b"])
    total, slot, act = opk.arena_bytes(ospec, P_F, P_B, cfg["M"], cfg["b"], cfg["precision"])
    assert (a["total"], a["slot_bytes"], a["act_bytes"]) == (total, slot, act)
    assert a["total"] <= cfg["budget"]
    # structure the paper states: forward packs cover the layers before the last
    # backward pack and are at least as large as backward packs
    assert (P_F[-1][1] if P_F else 0) == P_B[-1][0]
    if P_F and len(P_B) > 1:
        assert max(e - a_ for a_, e in P_F) >= max(e - a_ for a_, e in P_B[:-1])


@pytest.mark.parametrize("name", ["gpt2m", "gpt2xl", "bertl", "gpt6b7"])
def test_pack_count_search_matches_the_oracle_and_never_estimates_worse(name):
    """Algorithm 1's selection rule over the candidates Algorithm 2 produces: the
    searched plan equals the oracle's, its estimate equals the oracle's estimate,
    and it is no worse than the first feasible packing's."""
    cfg = synth.CONFIGS[name]
    spec, ospec = B.make_spec(cfg), oracle_spec(cfg)
    first = B.hmy_plan(spec, cfg["budget"], cfg["M"], cfg["b"])
    for link, rate in ((0, 0), (25000, 600000)):
        kw = dict(link_MBps=link or 40000, compute_GFLOPs=rate or 420000)
        s = B.hmy_plan(spec, cfg["budget"], cfg["M"], cfg["b"], search=64, link_MBps=link, compute_GFLOPs=rate)
        P_F, P_B = B.schedule_packs(s)
        want = opk.plan(ospec, cfg["budget"], cfg["M"], cfg["b"], cfg["precision"], search=64, **kw)
        assert (P_F, P_B) == want
        ns = B.hmy_estimate(spec, s, cfg["M"], cfg["b"], link, rate)
        assert ns == opk.estimate_iteration_ns(ospec, P_F, P_B, cfg["M"], cfg["b"], cfg["precision"],
                                               kw["link_MBps"], kw["compute_GFLOPs"])
        assert ns <= B.hmy_estimate(spec, first, cfg["M"], cfg["b"], link, rate)
        assert B.hmy_arena(spec, s, cfg["M"], cfg["b"])["total"] <= cfg["budget"]
        # planned for the Weight Update on the CPU: the schedule says so, plan and estimate equal the oracle's
        sh = B.hmy_plan(spec, cfg["budget"], cfg["M"], cfg["b"], search=64, link_MBps=link, compute_GFLOPs=rate,
                        update_site=B.HMY_UPDATE_ON_HOST)
        assert sh.update_site == B.HMY_UPDATE_ON_HOST
        P_Fh, P_Bh = B.schedule_packs(sh)
        assert (P_Fh, P_Bh) == opk.plan(ospec, cfg["budget"], cfg["M"], cfg["b"], cfg["precision"], search=64,
                                        update_on_host=True, **kw)
        nsh = B.hmy_estimate(spec, sh, cfg["M"], cfg["b"], link, rate)
        assert nsh == opk.estimate_iteration_ns(ospec, P_Fh, P_Bh, cfg["M"], cfg["b"], cfg["precision"],
                                                kw["link_MBps"], kw["compute_GFLOPs"], update_on_host=True)
        s.update_site = B.HMY_UPDATE_ON_HOST            # the device plan run with the update on the host
        assert nsh <= B.hmy_estimate(spec, s, cfg["M"], cfg["b"], link, rate)
        s.update_site = B.HMY_UPDATE_ON_DEVICE
        assert nsh <= ns                                # less traffic, never a longer estimate


def test_runtime_estimate_closed_forms():
    """Degenerate cases of the estimator that can be worked by hand: with an
    infinitely fast link the estimate is the sum of the visits' compute times; with
    infinitely fast compute it is the serial swap time of the dominant direction."""
    cfg = tiny_cfg(n_blocks=3, d_model=64, n_heads=2, d_ffn=128, seq_len=16, vocab=50, precision="bf16", M=2, b=2)
    spec, ospec = B.make_spec(cfg), oracle_spec(cfg)
    sched = B.make_schedule([2, 4], [2, 4, 5])
    prof = opk.layer_profile(ospec, 2, 2, "bf16")
    rate = 1000                                      # GFLOP/s = flops per ns
    flops = 2 * (sum(prof[l]["t_fwd"] for l in range(4)) + sum(prof[l]["t_bwd"] for l in range(5)))
    per_visit = [2 * sum(prof[l]["t_fwd"] for l in r) for r in (range(0, 2), range(2, 4))] + \
                [2 * sum(prof[l]["t_bwd"] for l in r) for r in (range(4, 5), range(2, 4), range(0, 2))]
    assert sum(per_visit) == flops
    fast_link = B.hmy_estimate(spec, sched, 2, 2, link_MBps=4_000_000_000, compute_GFLOPs=rate)
    assert abs(fast_link - sum(-(-f // rate) for f in per_visit)) <= 10     # + a few ns of (rounded-up) transfers
    n = sum(p["params"] for p in prof)
    slow = B.hmy_estimate(spec, sched, 2, 2, link_MBps=1, compute_GFLOPs=4_000_000_000)
    # device->host moves (12 + 2 + 4) B/param once; host->device moves 12 B/param of state + weights twice minus the last pack
    d2h_ns = 18 * n * 1000
    assert d2h_ns <= slow <= d2h_ns + 2 * 2 * n * 1000 + 12 * n * 1000 + 100
    # the update on the host: only the weights come in and only the 4 B/param gradient goes out; with a slow link
    # the weight loads (twice, minus the last pack) are the longer queue, the CPU (6 parameters/ns) comes after
    host = B.make_schedule([2, 4], [2, 4, 5], update_site=B.HMY_UPDATE_ON_HOST)
    slow_h = B.hmy_estimate(spec, host, 2, 2, link_MBps=1, compute_GFLOPs=4_000_000_000)
    n_last = prof[4]["params"]
    w_in_ns = 2 * (2 * n - n_last) * 1000
    assert w_in_ns <= slow_h <= w_in_ns + 4 * n * 1000 + n // 6 + 100
    fast_h = B.hmy_estimate(spec, host, 2, 2, link_MBps=4_000_000_000, compute_GFLOPs=rate)
    first_pack = prof[0]["params"] + prof[1]["params"]        # updated last: nothing left to hide its CPU time
    assert abs(fast_h - (fast_link + first_pack // 6)) <= 10


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


def test_planner_matches_oracle_on_random_small_models_and_budgets():
    rng = np.random.default_rng(0)
    n_checked = 0
    for _ in range(60):
        H = int(rng.choice([1, 2, 4]))
        dh = int(rng.choice([32, 64]))
        cfg = tiny_cfg(n_blocks=int(rng.integers(1, 9)), d_model=H * dh, n_heads=H,
                       d_ffn=int(rng.choice([64, 128, 512])), seq_len=int(rng.choice([8, 16, 64])),
                       vocab=int(rng.integers(17, 3000)), causal=int(rng.integers(0, 2)),
                       precision=str(rng.choice(["fp32", "bf16"])), M=int(rng.integers(1, 5)), b=int(rng.integers(1, 4)))
        spec, ospec = B.make_spec(cfg), oracle_spec(cfg)
        lo = one_layer_budget(cfg)
        prof = opk.layer_profile(ospec, cfg["M"], cfg["b"], cfg["precision"])
        hi = lo + sum(p["mem_bwd"] for p in prof)
        for budget in (lo // 2, lo, (lo + hi) // 2, int(lo + 0.3 * (hi - lo)), hi + 10 ** 6):
            want = opk.plan(ospec, budget, cfg["M"], cfg["b"], cfg["precision"])
            try:
                got = B.schedule_packs(B.hmy_plan(spec, budget, cfg["M"], cfg["b"]))
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

