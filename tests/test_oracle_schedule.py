"""Pins for the layer-pack-major driver, the swap-volume counts and the
balanced-time packing of the oracle."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import model as om
from oracle import packing as opk
from oracle import schedule as osch
from oracle import simulate as osim
from oracle import swapcount as osw
from paper_2202_01306_amd import synth
from tests.helpers import f64, oracle_spec, tiny_cfg


def all_packings(R):
    """Every way to cut 0..R into contiguous non-empty packs."""
    for mask in range(1 << (R - 1)):
        cuts = [i + 1 for i in range(R - 1) if mask >> i & 1]
        b = [0] + cuts + [R]
        yield list(zip(b[:-1], b[1:]))


# ---------------------------------------------------------------- schedule ---

@pytest.mark.parametrize("causal", [1, 0])
def test_layer_pack_major_is_bit_identical_to_microbatch_major(causal):
    """The paper's correctness claim (Section 5.4, "Correctness of Training"): the swapped, regrouped
    schedule gives exactly what ordinary training gives."""
    cfg = tiny_cfg(n_blocks=3, causal=causal, M=3, b=2)
    spec = oracle_spec(cfg)
    params = f64(synth.gen_params(cfg, 1, bench_init=False))
    m0, v0 = (f64(x) for x in synth.gen_adam_state(cfg, 1, zero=False))
    ids = synth.gen_tokens(cfg, 1)
    tg = synth.gen_targets(cfg, ids, 1)
    hp = om.AdamHP(step=10)
    ref = om.training_iteration(spec, params, ids, tg, m0, v0, hp)
    R = spec.n_layers   # 5
    tried = 0
    for P_B in all_packings(R):
        last_start = P_B[-1][0]
        fwd_opts = list(all_packings(last_start)) if last_start > 0 else [[]]
        for P_F in fwd_opts[::3] + fwd_opts[-1:]:
            out = osch.iteration_layer_pack_major(spec, params, ids, tg, P_F, P_B, m0, v0, hp)
            assert out["loss"] == ref["loss"] or abs(out["loss"] - ref["loss"]) < 1e-15
            for k in ("grads", "weights", "m", "v"):
                for name in params:
                    np.testing.assert_array_equal(out[k][name], ref[k][name], err_msg=f"{k}:{name}")
            tried += 1
    assert tried > 16


def test_distinct_forward_and_backward_microbatch_sizes_give_the_same_iteration():
    """Section 4.3.1: the configuration is a 4-tuple with its own microbatch size per pass (Algorithm 1 sweeps
    U_F and U_B separately).  Re-cutting the minibatch for the forward pass regroups rows, nothing else: with
    U_F = U_B the driver is the bit-identical one above; with another U_F every result agrees with the definition
    up to the rounding order inside the library's matrix products (1e-12 of each tensor's largest value), and the
    checkpoint volume is the same bytes cut differently."""
    cfg = tiny_cfg(n_blocks=3, M=3, b=4)
    spec = oracle_spec(cfg)
    params = f64(synth.gen_params(cfg, 2, bench_init=False))
    m0, v0 = (f64(x) for x in synth.gen_adam_state(cfg, 2, zero=False))
    ids = synth.gen_tokens(cfg, 2)
    tg = synth.gen_targets(cfg, ids, 2)
    hp = om.AdamHP(step=10)
    ref = om.training_iteration(spec, params, ids, tg, m0, v0, hp)
    for P_F, P_B in (([(0, 2), (2, 4)], [(0, 1), (1, 2), (2, 4), (4, 5)]), ([(0, 3)], [(0, 3), (3, 5)]),
                     ([], [(0, 5)]), ([(0, 1), (1, 4)], [(0, 2), (2, 3), (3, 4), (4, 5)])):
        same = osch.iteration_layer_pack_major(spec, params, ids, tg, P_F, P_B, m0, v0, hp, U_F=4)
        for k in ("grads", "weights", "m", "v"):
            for name in params:
                np.testing.assert_array_equal(same[k][name], ref[k][name])
        for U_F in (1, 2, 3, 6, 12):
            out = osch.iteration_layer_pack_major(spec, params, ids, tg, P_F, P_B, m0, v0, hp, U_F=U_F)
            assert abs(out["loss"] - ref["loss"]) < 1e-13 * abs(ref["loss"])
            for k in ("grads", "weights", "m", "v"):
                for name in params:
                    scale = max(np.abs(ref[k][name]).max(), 1e-300)
                    assert np.abs(out[k][name] - ref[k][name]).max() <= 1e-12 * scale, (U_F, k, name)
            M_F = 12 // U_F
            for prec in ("fp32", "bf16"):
                cf = osw.closed_form(spec, P_F, P_B, 3, 4, prec, M_F=M_F, b_F=U_F)
                assert cf == osw.closed_form(spec, P_F, P_B, 3, 4, prec)
                assert cf == osw.ledger(spec, P_F, P_B, 3, 4, prec, M_F=M_F, b_F=U_F)
    with pytest.raises(ValueError):
        osch.iteration_layer_pack_major(spec, params, ids, tg, [(0, 3)], [(0, 3), (3, 5)], m0, v0, hp, U_F=5)
    with pytest.raises(ValueError):
        osw.closed_form(spec, [(0, 3)], [(0, 3), (3, 5)], 3, 4, "fp32", M_F=5, b_F=2)


def test_microbatch_major_over_packs_is_bit_identical_too():
    """The comparison order of Section 3 (every microbatch on its own through all packs,
    gradients summed across microbatches, update after the last one) is ordinary
    training as well: same loss, gradients and updated state, bit for bit."""
    cfg = tiny_cfg(n_blocks=3, M=3, b=2)
    spec = oracle_spec(cfg)
    params = f64(synth.gen_params(cfg, 2, bench_init=False))
    m0, v0 = (f64(x) for x in synth.gen_adam_state(cfg, 2, zero=False))
    ids = synth.gen_tokens(cfg, 2)
    tg = synth.gen_targets(cfg, ids, 2)
    hp = om.AdamHP(step=3)
    ref = om.training_iteration(spec, params, ids, tg, m0, v0, hp)
    for P_F, P_B in (([(0, 1), (1, 2), (2, 3), (3, 4)], [(0, 1), (1, 2), (2, 3), (3, 4), (4, 5)]),
                     ([(0, 3)], [(0, 2), (2, 3), (3, 5)]), ([], [(0, 5)])):
        tasks = osch.task_list_microbatch_major(spec, P_F, P_B, 3)
        assert [t.index for t in tasks] == list(range(len(tasks)))
        assert sum(t.kind == "A" for t in tasks) == len(P_B) and all(t.mb == 2 for t in tasks if t.kind == "A")
        # per microbatch: every forward pack, then every backward pack in reverse
        for mb in range(3):
            mine = [t for t in tasks if t.mb == mb and t.kind != "A"]
            assert [t.pack for t in mine] == list(P_F) + list(reversed(P_B))
        out = osch.iteration_layer_pack_major(spec, params, ids, tg, P_F, P_B, m0, v0, hp, order="microbatch_major")
        assert abs(out["loss"] - ref["loss"]) < 1e-15
        for k in ("grads", "weights", "m", "v"):
            for name in params:
                np.testing.assert_array_equal(out[k][name], ref[k][name], err_msg=f"{k}:{name}")


def test_task_list_order_follows_algorithm_3():
    spec = om.Spec(4, 8, 2, 16, 4, 16)
    P_B = [(0, 2), (2, 4), (4, 6)]
    P_F = [(0, 3), (3, 4)]
    tl = osch.task_list(spec, P_F, P_B)
    assert [(t.kind, t.pack) for t in tl] == [
        ("F", (0, 3)), ("F", (3, 4)),
        ("B", (4, 6)), ("A", (4, 6)), ("B", (2, 4)), ("A", (2, 4)), ("B", (0, 2)), ("A", (0, 2))]
    assert [t.index for t in tl] == list(range(8))
    assert tl[0].stash_out_layers == [2] and tl[1].stash_out_layers == []
    assert tl[4].stash_in_layer == 2 and tl[6].stash_in_layer is None and tl[2].stash_in_layer is None


def test_bad_packs_are_rejected():
    spec = om.Spec(2, 8, 2, 16, 4, 16)
    with pytest.raises(ValueError):
        osch.check_packs(spec, [], [(0, 2), (3, 4)])
    with pytest.raises(ValueError):
        osch.check_packs(spec, [(0, 1)], [(0, 2), (2, 4)])
    with pytest.raises(ValueError):
        osch.check_packs(spec, [], [(0, 3)])
    osch.check_packs(spec, [(0, 1), (1, 2)], [(0, 2), (2, 4)])


# -------------------------------------------------------------- swap bytes ---

def test_residency_machine_reproduces_the_papers_weight_volumes():
    """Section 3, 'Intuitive Example': one layer fits; equal layers.
    Per-GPU swap: (4m+2)|W|.  Harmony: 3|W|."""
    for R, m in itertools.product((1, 2, 6, 13), (1, 2, 5)):
        pack_bytes = [1000] * R
        W = sum(pack_bytes)
        i, o = osw.residency_machine(osw.steps_microbatch_major(R, m, True), pack_bytes, True)
        assert i + o == osw.paper_W_volume_per_gpu_swap_dp(m, 1, W) == (4 * m + 2) * W
        i, o = osw.residency_machine(osw.steps_layer_pack_major(R, m, False), pack_bytes, False)
        assert (i, o) == (2 * W, W)
        assert i + o == osw.paper_W_volume_harmony_dp(1, W) == 3 * W
        # jit-compute shares the last pack between the passes
        i, o = osw.residency_machine(osw.steps_layer_pack_major(R, m, True), pack_bytes, False)
        assert (i, o) == (2 * W - pack_bytes[-1], W)


def _golden_rows(name):
    path = os.path.join(os.path.dirname(__file__), "golden", name)
    return [l.split() for l in open(path) if l.strip() and not l.startswith("#")]


def test_paper_stated_swap_volumes():
    """tests/golden/paper_swap_volumes.txt holds the volumes the paper states (Section 3 'Intuitive Example',
    appendix 'Additional Swap Analysis'), typed from its text.  The residency machine, which knows nothing of
    those formulas, reproduces every single-GPU row; the N-GPU rows are N independent copies (data parallelism)
    or one copy (pipeline); the oracle's own statement of the formulas agrees with all of them."""
    rows = _golden_rows("paper_swap_volumes.txt")
    assert len(rows) == 15
    R = 5
    unit = [700] * R               # equal layers, one layer fits: the setting of the paper's example
    total = sum(unit)
    for kind, scheme, m, N, want in rows:
        m, N, want = int(m), int(N), int(want)
        if kind == "W" and scheme in ("per_gpu_swap_dp", "per_gpu_swap_pp"):
            i, o = osw.residency_machine(osw.steps_microbatch_major(R, m, True), unit, True)
            copies = N if scheme.endswith("_dp") else 1
            assert copies * (i + o) == want * total
            if scheme.endswith("_dp"):
                assert osw.paper_W_volume_per_gpu_swap_dp(m, N, total) == want * total
        elif kind == "W":
            i, o = osw.residency_machine(osw.steps_layer_pack_major(R, m, False), unit, False)
            copies = N if scheme.endswith("_dp") else 1
            assert copies * (i + o) == want * total
            if scheme.endswith("_dp"):
                assert osw.paper_W_volume_harmony_dp(N, total) == want * total
        elif kind == "dW":
            # the gradient buffer in a virtual memory that writes back all it evicts: resident only in backward
            # passes (m of them, each swapping every pack in and out) and in the update phase (once more each way)
            steps = []
            for _ in range(m):
                steps += [(p, True) for p in reversed(range(R))] + [osw.FLUSH]
            steps += [(p, True) for p in range(R)]
            i, o = osw.residency_machine(steps, unit, True)
            assert N * (i + o) == want * total == osw.paper_dW_volume_per_gpu_swap_dp(m, N, total)
        else:
            i, o = osw.residency_machine([(p, True) for p in range(R)], unit, True)
            assert N * (i + o) == want * total == osw.paper_K_volume(N, total)


def test_paper_stated_workloads():
    """tests/golden/paper_workloads.txt: layer counts, sequence lengths and sizes as Section 5.1 lists them; the
    synthetic stand-ins have those shapes, and their parameter counts truncate to the sizes the paper prints."""
    for name, cfg_name, layers, seq, size in _golden_rows("paper_workloads.txt"):
        cfg = synth.CONFIGS[cfg_name]
        assert cfg["n_blocks"] == int(layers) and cfg["seq_len"] == int(seq), name
        if size != "-":
            spec = oracle_spec(cfg)
            n = sum(om.layer_param_count(spec, l) for l in range(spec.n_layers)) - cfg["vocab"] * cfg["d_model"]
            assert f"{math.floor(n / 1e8) / 10:.1f}B" == size, (name, n)     # tied head, as the models are published


@pytest.mark.parametrize("precision", ["fp32", "bf16"])
def test_closed_form_equals_ledger_equals_machine_on_every_packing(precision):
    spec = om.Spec(4, 8, 2, 24, 4, 16)      # R = 6, unequal layers
    R = spec.n_layers
    w_c, k_B, g_B = osw.bytes_per_param(precision)
    pc = [om.layer_param_count(spec, l) for l in range(R)]
    for M, b in ((1, 1), (3, 2)):
        for P_B in all_packings(R):
            last_start = P_B[-1][0]
            for P_F in (list(all_packings(last_start)) if last_start else [[]]):
                cf = osw.closed_form(spec, P_F, P_B, M, b, precision)
                lg = osw.ledger(spec, P_F, P_B, M, b, precision)
                assert cf == lg
                # weights, from first principles: forward packs then backward packs
                packs = list(P_F) + list(P_B)
                steps = [(i, False) for i in range(len(P_F)) for _ in range(M)]
                for j in reversed(range(len(P_B))):
                    steps += [(len(P_F) + j, False)] * M + [(len(P_F) + j, True)]
                pb = [w_c * sum(pc[a:e]) for (a, e) in packs]
                i, o = osw.residency_machine(steps, pb, False)
                assert (i, o) == (cf["h2d"]["W"], cf["d2h"]["W"])
                # microbatch-major brings the weights in exactly M times as often
                mm = osw.closed_form_microbatch_major(spec, P_F, P_B, M, b, precision)
                assert mm["h2d"]["W"] == M * cf["h2d"]["W"]
                # optimizer state: in and out once (appendix), gradients never come in
                K = k_B * sum(pc)
                assert cf["h2d"]["K"] + cf["d2h"]["K"] == osw.paper_K_volume(1, K)
                assert cf["h2d"]["dW"] == 0 and cf["d2h"]["dW"] == g_B * sum(pc)
                assert cf["h2d"]["sX"] == cf["d2h"]["sX"] == \
                    M * b * spec.seq_len * spec.d_model * w_c * max(len(P_B) - 2, 0)


@pytest.mark.parametrize("precision", ["fp32", "bf16"])
def test_microbatch_major_volumes_closed_form_ledger_machine(precision):
    """Closed form = walk over the microbatch-major task list = residency machine, on
    every packing; and the distance to the paper's own dW count is exactly the three
    transfers the readings remove (no first swap-in, no swap-in and no second swap-out
    around a separate update phase)."""
    spec = om.Spec(4, 8, 2, 24, 4, 16)      # R = 6, unequal layers
    R = spec.n_layers
    w_c, k_B, g_B = osw.bytes_per_param(precision)
    pc = [om.layer_param_count(spec, l) for l in range(R)]
    for M, b in ((1, 1), (2, 1), (4, 2)):
        for P_B in all_packings(R):
            last_start = P_B[-1][0]
            fwd_opts = list(all_packings(last_start)) if last_start else [[]]
            for P_F in fwd_opts[::2] + fwd_opts[-1:]:
                cf = osw.closed_form_microbatch_major(spec, P_F, P_B, M, b, precision)
                assert cf == osw.ledger_microbatch_major(spec, P_F, P_B, M, b, precision)
                lpm = osw.closed_form(spec, P_F, P_B, M, b, precision)
                for kind in ("K", "sX", "ids"):
                    assert cf["h2d"][kind] == lpm["h2d"][kind] and cf["d2h"][kind] == lpm["d2h"][kind]
                assert cf["d2h"]["W"] == lpm["d2h"]["W"]
                # weights from first principles: one pack resident at a time, clean ones dropped
                packs = list(P_F) + list(P_B)
                one_mb = [(i, False) for i in range(len(P_F))] + \
                         [(len(P_F) + j, False) for j in reversed(range(len(P_B)))]
                steps = []
                for mb in range(M):
                    steps += one_mb if mb < M - 1 else one_mb[:len(P_F)]
                    if mb < M - 1:
                        steps.append(osw.FLUSH)     # the first forward pack of the next microbatch comes in anew
                for j in reversed(range(len(P_B))):
                    steps += [(len(P_F) + j, False), (len(P_F) + j, True)]
                i, o = osw.residency_machine(steps, [w_c * sum(pc[a:e]) for (a, e) in packs], False)
                assert (i, o) == (cf["h2d"]["W"], cf["d2h"]["W"])
                # gradient buffers: written by every backward task, one resident at a time
                gsteps = []
                for mb in range(M):
                    gsteps += [(j, True) for j in reversed(range(len(P_B)))] + [osw.FLUSH]
                gi, go = osw.residency_machine(gsteps, [g_B * sum(pc[a:e]) for (a, e) in P_B], False)
                dW = g_B * sum(pc)
                assert go == cf["d2h"]["dW"] == M * dW
                assert gi - dW == cf["h2d"]["dW"]          # the machine also "reads" the first, all-zero buffer
                assert cf["h2d"]["dW"] + cf["d2h"]["dW"] == osw.paper_dW_volume_per_gpu_swap_dp(M, 1, dW) - 3 * dW


def test_update_on_host_moves_only_the_gradient():
    """Weight Update on the CPU (Section 4.4): K and the updated W stay where they live,
    so the link carries W in (two passes), the checkpoints, and dW out once; everything
    else equals the on-device count.  Closed form = ledger, both orders."""
    spec = om.Spec(4, 8, 2, 24, 4, 16)
    R = spec.n_layers
    for precision in ("fp32", "bf16"):
        w_c, k_B, g_B = osw.bytes_per_param(precision)
        P = sum(om.layer_param_count(spec, l) for l in range(R))
        for M, b in ((1, 1), (3, 2)):
            for P_B in list(all_packings(R))[::3]:
                last_start = P_B[-1][0]
                P_F = [(0, last_start)] if last_start else []
                dev = osw.closed_form(spec, P_F, P_B, M, b, precision)
                host = osw.closed_form(spec, P_F, P_B, M, b, precision, update_on_host=True)
                assert host == osw.ledger(spec, P_F, P_B, M, b, precision, update_on_host=True)
                assert host["h2d"]["K"] == host["d2h"]["K"] == host["d2h"]["W"] == 0
                assert host["d2h"]["dW"] == g_B * P
                saved = sum(dev[d][k] - host[d][k] for d in ("h2d", "d2h") for k in osw.KINDS)
                assert saved == (2 * k_B + w_c) * P       # K both ways and W out
                mm = osw.closed_form_microbatch_major(spec, P_F, P_B, M, b, precision, update_on_host=True)
                assert mm == osw.ledger_microbatch_major(spec, P_F, P_B, M, b, precision, update_on_host=True)
                assert mm["h2d"]["K"] == mm["d2h"]["K"] == mm["d2h"]["W"] == 0 and mm["d2h"]["dW"] == M * g_B * P


def test_gradients_dropped_on_the_device_is_the_papers_own_count():
    """Section 3, second optimisation: the update consumes dW while it is resident, so in
    the paper dW never crosses the link.  With export_gradients=False the closed form and
    the ledger say so; W, K and checkpoints are untouched, and with the update on the host
    the switch changes nothing (there the gradient is the update's input).  Microbatch-major:
    M - 1 out and M - 1 in remain (the parking between microbatches)."""
    spec = om.Spec(4, 8, 2, 24, 4, 16)
    R = spec.n_layers
    for precision in ("fp32", "bf16"):
        w_c, k_B, g_B = osw.bytes_per_param(precision)
        P = sum(om.layer_param_count(spec, l) for l in range(R))
        for M, b in ((1, 1), (3, 2)):
            for P_B in list(all_packings(R))[::3]:
                last_start = P_B[-1][0]
                P_F = [(0, last_start)] if last_start else []
                args = (spec, P_F, P_B, M, b, precision)
                exp, drop = osw.closed_form(*args), osw.closed_form(*args, export_gradients=False)
                assert drop == osw.ledger(*args, export_gradients=False)
                assert drop["d2h"]["dW"] == 0 and drop["h2d"]["dW"] == 0
                assert exp["d2h"]["dW"] - drop["d2h"]["dW"] == g_B * P
                for d in ("h2d", "d2h"):
                    for k in osw.KINDS:
                        if (d, k) != ("d2h", "dW"):
                            assert exp[d][k] == drop[d][k]
                assert osw.closed_form(*args, update_on_host=True, export_gradients=False) == \
                    osw.closed_form(*args, update_on_host=True) == \
                    osw.ledger(*args, update_on_host=True, export_gradients=False)
                mm = osw.closed_form_microbatch_major(*args, export_gradients=False)
                assert mm == osw.ledger_microbatch_major(*args, export_gradients=False)
                assert mm["d2h"]["dW"] == mm["h2d"]["dW"] == (M - 1) * g_B * P
                assert osw.closed_form_microbatch_major(*args, update_on_host=True, export_gradients=False) == \
                    osw.ledger_microbatch_major(*args, update_on_host=True, export_gradients=False) == \
                    osw.closed_form_microbatch_major(*args, update_on_host=True)


def test_resident_optimizer_state_leaves_the_link_alone():
    """Optimizer state pinned on the device (Algorithm 3's GPU-pinned channel): for P_res resident parameters
    the appendix's K volume 2 |K| shrinks by their share both ways; the first iteration still reads them once;
    W, dW, checkpoints do not change; nothing to pin when the update runs on the host."""
    spec = om.Spec(4, 8, 2, 24, 4, 16)
    R = spec.n_layers
    P = sum(om.layer_param_count(spec, l) for l in range(R))
    for precision in ("fp32", "bf16"):
        w_c, k_B, g_B = osw.bytes_per_param(precision)
        for M, b in ((1, 1), (3, 2)):
            for P_B in list(all_packings(R))[::5]:
                last_start = P_B[-1][0]
                P_F = [(0, last_start)] if last_start else []
                args = (spec, P_F, P_B, M, b, precision)
                base = osw.closed_form(*args)
                assert base["h2d"]["K"] + base["d2h"]["K"] == osw.paper_K_volume(1, k_B * P)
                for P_res in (0, 1, P // 3, P):
                    for cf in (osw.closed_form, osw.closed_form_microbatch_major):
                        plain = cf(*args)
                        steady = cf(*args, resident_K_params=P_res)
                        first = cf(*args, resident_K_params=P_res, resident_K_loaded=False)
                        assert steady["h2d"]["K"] == steady["d2h"]["K"] == k_B * (P - P_res)
                        assert first["h2d"]["K"] == k_B * P and first["d2h"]["K"] == k_B * (P - P_res)
                        for d in ("h2d", "d2h"):
                            for k in osw.KINDS:
                                if k != "K":
                                    assert plain[d][k] == steady[d][k] == first[d][k]
                        assert cf(*args, update_on_host=True, resident_K_params=P_res) == cf(*args, update_on_host=True)
                with pytest.raises(ValueError):
                    osw.closed_form(*args, resident_K_params=P + 1)
                # the closed form's residency terms against a walk that knows nothing of them: the ledger visits
                # the update tasks piece by piece and skips the optimizer state of pieces marked resident
                for chunk in (7, 100, 10 ** 6):
                    pieces = osw.update_chunks(spec, P_B, chunk)
                    assert sum(n for (_, _, n) in pieces) == P
                    for n_res in (0, 1, len(pieces) // 2, len(pieces)):
                        chosen = pieces[len(pieces) - n_res:]         # the pieces updated last
                        res_set = {(pack, c) for (pack, c, _) in chosen}
                        P_res = sum(n for (_, _, n) in chosen)
                        for loaded in (True, False):
                            for export in (True, False):
                                assert osw.ledger(*args, export_gradients=export, chunk_params=chunk, resident=res_set,
                                                  resident_loaded=loaded) == \
                                    osw.closed_form(*args, export_gradients=export, resident_K_params=P_res,
                                                    resident_K_loaded=loaded)


def test_weight_volume_reduces_to_3W_when_last_pack_is_counted_twice():
    spec = om.Spec(3, 8, 2, 16, 4, 16)
    P_B = [(0, 2), (2, 4), (4, 5)]
    P_F = [(0, 4)]
    cf = osw.closed_form(spec, P_F, P_B, 4, 2, "fp32")
    W = 4 * sum(om.layer_param_count(spec, l) for l in range(5))
    W_last = 4 * om.layer_param_count(spec, 4)
    assert cf["h2d"]["W"] + cf["d2h"]["W"] + W_last == osw.paper_W_volume_harmony_dp(1, W)


def test_parameter_counts_match_the_workload_table():
    """p_blk = 4d^2 + 2df + 9d + f; GPT-2-medium ~ 355 M parameters."""
    cfg = synth.CONFIGS["gpt2m"]
    spec = oracle_spec(cfg)
    d, f = 1024, 4096
    assert om.layer_param_count(spec, 1) == 4 * d * d + 2 * d * f + 9 * d + f == 12_596_224
    total = sum(om.layer_param_count(spec, l) for l in range(spec.n_layers))
    assert total - 50257 * d == 354_823_168        # tied-head count of GPT-2 medium
    assert list(om.param_shapes(spec).items()) == list(synth.shape_table(cfg).items())


# ----------------------------------------------------------------- packing ---

def test_equal_layers_split_evenly():
    assert opk.balanced_time_packing([5] * 4, [10] * 4, 20) == [(0, 2), (2, 4)]
    # ties are exact: 6 equal layers into 4 packs
    packs = opk.balanced_time_packing([7] * 6, [10] * 6, 19)      # one layer per pack would be 6
    assert packs == [(0, 1), (1, 2), (2, 3), (3, 4), (4, 5), (5, 6)]
    packs = opk.balanced_time_packing([7] * 6, [10] * 6, 20)
    assert packs == [(0, 2), (2, 4), (4, 6)]


def test_packing_properties_on_random_profiles():
    rng = np.random.default_rng(0)
    for _ in range(300):
        R = int(rng.integers(1, 14))
        t = [int(x) for x in rng.integers(1, 100, R)]
        m = [int(x) for x in rng.integers(1, 50, R)]
        alpha = int(rng.integers(max(m), 4 * max(m) + 1))
        packs = opk.balanced_time_packing(t, m, alpha)
        assert packs is not None
        assert packs[0][0] == 0 and packs[-1][1] == R
        assert all(a < e for a, e in packs)
        assert all(p[1] == q[0] for p, q in zip(packs, packs[1:]))
        assert all(sum(m[a:e]) <= alpha for a, e in packs)
        S_min = max(1, -(-sum(m) // alpha))
        assert len(packs) >= S_min or len(packs) >= 1
        # first feasible S is returned: every smaller S (from S_min) has an over-full pack
        for S in range(S_min, R + 1):
            cand = opk.packs_from_cuts(opk.split_points(t, S), R)
            if all(sum(m[a:e]) <= alpha for a, e in cand):
                assert cand == packs
                break
        else:   # no balanced split fits: one layer per pack
            assert packs == [(j, j + 1) for j in range(R)]


def test_infeasible_when_one_layer_exceeds_capacity():
    assert opk.balanced_time_packing([1, 1, 1], [5, 50, 5], 49) is None
    assert opk.balanced_time_packing([], [], 10) == []


def test_paper_table_of_layer_packs_has_the_structure_the_planner_builds():
    """tests/golden/paper_detailed_packs.txt (appendix table 'Detailed scheduling result').  What does not depend
    on the paper's measured layer times: packs are contiguous and cover the model; the forward packs cover exactly
    the layers before the last backward pack (the opening steps of Algorithm 2); over the uniform transformer
    layers pack sizes differ by at most one; and Algorithm 2 on equal layers with the table's largest pack as
    capacity gives the same NUMBER of packs of each size (which ones are the shorter packs is the paper's
    profile's doing)."""
    table = {}
    for row in _golden_rows("paper_detailed_packs.txt"):
        table[(row[0], row[1])] = [(int(a), int(b) + 1) for a, b in (p.split("-") for p in row[2:])]
    assert set(table) == {("BERT96", "P_F"), ("BERT96", "P_B"), ("GPT2", "P_F"), ("GPT2", "P_B")}
    for model in ("BERT96", "GPT2"):
        P_F, P_B = table[(model, "P_F")], table[(model, "P_B")]
        for packs in (P_F, P_B):
            assert packs[0][0] == 0 and all(p[1] == q[0] for p, q in zip(packs, packs[1:]))
        assert P_F[-1][1] == P_B[-1][0] == opk.forward_layers_given_backward(P_B)
        for packs in (P_F, P_B[:-1]):                          # the last backward pack also holds the output layers
            sizes = [e - a for a, e in packs]
            assert max(sizes) - min(sizes) <= 1
            n = packs[-1][1]
            mine = opk.balanced_time_packing([10] * n, [1] * n, max(sizes))
            assert sorted(e - a for a, e in mine) == sorted(sizes), (model, sizes)


def test_uniform_transformer_layers_give_pack_sizes_differing_by_at_most_one():
    """Shape of the paper's Table 'detailed scheduling result': BERT96's forward
    packs are 21 packs of 4 layers and 3 packs of 3 over 93 layers; GPT2's
    backward packs over blocks are 16 packs of 3 over 48 layers.
    (Exact positions depend on the paper's measured profiles: unpinned.)"""
    # 93 equal layers, capacity of 4 layers
    packs = opk.balanced_time_packing([10] * 93, [1] * 93, 4)
    sizes = [e - a for a, e in packs]
    assert len(packs) == 24 and sorted(set(sizes)) == [3, 4]
    assert sizes.count(4) == 21 and sizes.count(3) == 3
    packs = opk.balanced_time_packing([10] * 48, [1] * 48, 3)
    assert [e - a for a, e in packs] == [3] * 16
    packs = opk.balanced_time_packing([10] * 48, [1] * 48, 5)
    sizes = [e - a for a, e in packs]
    assert len(packs) == 10 and sizes.count(5) == 8 and sizes.count(4) == 2


def test_a_long_layer_gets_its_own_pack_and_empty_packs_are_dropped():
    t = [1, 1, 100, 1, 1]
    packs = opk.balanced_time_packing(t, [10] * 5, 25)
    assert packs is not None and all(10 * (e - a) <= 25 for a, e in packs)
    assert all(e > a for a, e in packs)
    assert packs[0][0] == 0 and packs[-1][1] == 5


def test_forward_packing_covers_layers_before_last_backward_pack():
    P_B = [(0, 3), (3, 6), (6, 8)]
    n = opk.forward_layers_given_backward(P_B)
    assert n == 6
    P_F = opk.balanced_time_packing([4] * n, [2] * n, 12)
    assert P_F == [(0, 6)]
    # forward footprints are smaller, so forward packs are at least as large
    assert max(e - a for a, e in P_F) >= max(e - a for a, e in P_B[:-1])


# -------------------------------------------------------------- simulation ---
# The event-driven estimate of an iteration (Section 4.3.1, Runtime Estimator), pinned by
# schedules walked by hand.  Toy model: embedding 160, blocks 736, head 144 parameters
# (d = 8, f = 24, s = 4, V = 16); fp32 (4 B weights, 8 B optimizer state, 4 B exported
# gradient per parameter); two microbatches; a checkpoint of 64 bytes per microbatch.
from fractions import Fraction as Fr


def _toy(n_blocks):
    spec = om.Spec(n_blocks, 8, 2, 24, 4, 16)
    assert [om.layer_param_count(spec, l) for l in range(spec.n_layers)] == [160] + [736] * n_blocks + [144]
    return spec


def _sim(spec, P_F, P_B, t_fwd, t_bwd, slots=3, distance=1, host=False, n_in=Fr(1, 64), n_out=Fr(1, 64), **kw):
    ops = osim.iteration_ops(spec, P_F, P_B, t_fwd, t_bwd, 2, 2, 64, 64, 4, 8, 4, n_in, n_out, slots=slots,
                             distance=distance, update_on_host=host, host_ns_per_param=Fr(1, 8), **kw)
    return osim.run(ops)


def test_generic_simulator_on_a_three_operation_example():
    """Two resources by hand: b waits for a; c shares a's resource and queues behind it;
    d may not end before c although it is shorter."""
    ops = [osim.Op("a", "x", Fr(5)), osim.Op("c", "x", Fr(7)), osim.Op("b", "y", Fr(2), after_end=["a"]),
           osim.Op("d", "y", Fr(1), after_start=["c"], not_before_end=["c"])]
    assert osim.run(ops) == {"a": (0, 5), "c": (5, 12), "b": (5, 7), "d": (7, 12)}
    with pytest.raises(AssertionError):
        osim.run([osim.Op("a", "x", Fr(1), after_end=["b"]), osim.Op("b", "y", Fr(1), after_end=["a"])])


def test_simulated_iteration_three_visits_worked_by_hand():
    """P_F = [0,2), P_B = [0,2) [2,4); link 1/64 ns per byte both ways.
    W0 = (160+736)*4/64 = 56, C0 = 2*(1+10) = 22; W1 = (736+144)/16 = 55, C1 = 2*(30+12) = 84,
    K1 = 880*8/64 = 110, Out1 = 880*16/64 = 220; W2 = 56, C2 = 2*(3+30) = 66, K2 = 112, Out2 = 224.
    W0 0-56; C0 56-78; W1 (asked at 56) 56-111; C1 111-195; W2 (asked at 111) 111-167;
    K1 (asked at 195) 195-305; Out1 195-415; C2 195-261; K2 305-417; Out2 415-639."""
    t = _sim(_toy(2), [(0, 2)], [(0, 2), (2, 4)], [1, 10, 10, 4], [3, 30, 30, 12])
    want = {"W0": (0, 56), "C0": (56, 78), "W1": (56, 111), "C1": (111, 195), "W2": (111, 167), "K1": (195, 305),
            "Out1": (195, 415), "C2": (195, 261), "K2": (305, 417), "Out2": (415, 639)}
    assert t == want
    # two slots change nothing here: the slot of visit 2 was a forward visit's, free since 78
    assert _sim(_toy(2), [(0, 2)], [(0, 2), (2, 4)], [1, 10, 10, 4], [3, 30, 30, 12], slots=2) == want


def test_simulated_iteration_with_checkpoints_and_host_update_worked_by_hand():
    """P_F = [0,3), four one-layer backward packs: checkpoints at layers 1 and 2.
    Device update, compute-bound (times 10/100/100/40 forward, 30/300/300/120 backward):
    W0 = 1632*4/64 = 102; C0 = 2*210 = 420; Sout0 = 2 checkpoints * 2 * 64/64 = 4; W1 = 9, C1 = 240, K1 = 18,
    Out1 = 36; visits 2, 3: W 46, C 600, K 92, Out 184, Sin 2; visit 4: W 10, C 60, K 20, Out 40.
    W0 0-102; C0 102-522; Sout0 102-106; W1 102-111; C1 522-762; W2 522-568; K1 762-780; Out1 762-798;
    C2 762-1362; Sin2 780-782; W3 782-828; K2 1362-1454; Out2 1362-1546; C3 1362-1962; Sin3 1454-1456;
    W4 1456-1466; K3 1962-2054; Out3 1962-2146; C4 1962-2022; K4 2054-2074; Out4 2146-2186."""
    spec = _toy(2)
    P_F, P_B = [(0, 3)], [(0, 1), (1, 2), (2, 3), (3, 4)]
    t = _sim(spec, P_F, P_B, [10, 100, 100, 40], [30, 300, 300, 120])
    assert t["Sout0"] == (102, 106) and t["Sin2"] == (780, 782) and t["W3"] == (782, 828) and t["Sin3"] == (1454, 1456)
    assert t["K3"] == (1962, 2054) and t["Out3"] == (1962, 2146) and t["C4"] == (1962, 2022)
    assert max(e for _, e in t.values()) == t["Out4"][1] == 2186
    # the update on the CPU (backward times 30/200/200/120, CPU at 8 parameters per ns): only the gradient leaves
    # Out1 = 144*4/64 = 9, Cpu1 = 18; Out 46 and Cpu 92 for the blocks; Out4 = 10, Cpu4 = 20
    # C1 522-762; Out1 762-771; Cpu1 771-789; C2 762-1162; Out2 1162-1208; Cpu2 1208-1300; C3 1162-1562;
    # Out3 1562-1608; Cpu3 1608-1700; C4 1562-1622; Out4 1622-1632; Cpu4 1700-1720
    h = _sim(spec, P_F, P_B, [10, 100, 100, 40], [30, 200, 200, 120], host=True)
    assert "K1" not in h and h["Out2"] == (1162, 1208) and h["Cpu3"] == (1608, 1700) and h["Cpu4"] == (1700, 1720)
    assert max(e for _, e in h.values()) == 1720


def test_simulated_visit_waits_for_its_checkpoints_worked_by_hand():
    """The schedule of the test above with short backward visits behind a slow incoming link (1/16 ns per byte:
    W0 = 408, W1 = 36, block W 184, W4 = 40; K1 = 72, block K 368, K4 = 80; Sin = 2*64/16 = 8; outgoing as before).
    Backward times 30/20/20/120: C2 = C3 = 40 alone, but the checkpoints they start from queue behind the
    optimizer state of the update before.
    W0 0-408; C0 408-828; W1 408-444; C1 828-1068; W2 828-1012; K1 1068-1140; Out1 1068-1140;
    C2 starts 1068, Sin2 (behind K1) 1140-1148, so C2 ends 1148, not 1108; W3 1148-1332; K2 1332-1700; Out2 1148-1700;
    C3 starts 1332, Sin3 (behind K2) 1700-1708, so C3 ends 1708; W4 1708-1748; K3 1748-2116; Out3 1708-2116;
    C4 1748-1808; K4 2116-2196; Out4 2116-2196."""
    spec = _toy(2)
    t = _sim(spec, [(0, 3)], [(0, 1), (1, 2), (2, 3), (3, 4)], [10, 100, 100, 40], [30, 20, 20, 120], n_in=Fr(1, 16))
    assert t["K1"] == (1068, 1140) and t["Sin2"] == (1140, 1148) and t["C2"] == (1068, 1148)
    assert t["W3"] == (1148, 1332) and t["K2"] == (1332, 1700) and t["Out2"] == (1148, 1700)
    assert t["Sin3"] == (1700, 1708) and t["C3"] == (1332, 1708) and t["W4"] == (1708, 1748)
    assert t["C4"] == (1748, 1808) and t["Out4"] == (2116, 2196) and max(e for _, e in t.values()) == 2196


def test_simulated_iteration_two_slots_against_three_worked_by_hand():
    """Seven visits (P_F = [0,5), six one-layer backward packs), device->host at 1/32 ns per byte:
    W0 = 3104*4/64 = 194, C0 = 2*410 = 820, Sout0 = 4*2*64/32 = 16; visit 1: W 9, C 240, K 18, Out 144*16/32 = 72;
    visits 2..5: W 46, C 400, K 92, Out 368, Sin 2; visit 6: W 10, C 60, K 20, Out 80.
    Two slots: W4 needs visit 2's slot, which Out2 leaves at 2022, so C4 starts at 2068 instead of 2054 and
    everything behind it is 14 later: 3316 against 3302 with three slots (W4 at 1748, visit 1's slot)."""
    spec = _toy(4)
    P_F, P_B = [(0, 5)], [(i, i + 1) for i in range(6)]
    tf, tb = [10, 100, 100, 100, 100, 40], [30, 200, 200, 200, 200, 120]
    two = _sim(spec, P_F, P_B, tf, tb, slots=2, n_out=Fr(1, 32))
    assert two["W3"] == (1326, 1372) and two["W4"] == (2022, 2068) and two["K3"] == (2068, 2160)
    assert two["C4"] == (2068, 2468) and two["W6"] == (2836, 2846) and two["Out6"] == (3236, 3316)
    three = _sim(spec, P_F, P_B, tf, tb, slots=3, n_out=Fr(1, 32))
    assert three["W3"] == (1274, 1320) and three["W4"] == (1748, 1794) and three["C4"] == (2054, 2454)
    assert max(e for _, e in three.values()) == 3302 and max(e for _, e in two.values()) == 3316
    for slots, distance in ((3, 2), (4, 1), (4, 2), (4, 3)):
        assert max(e for _, e in _sim(spec, P_F, P_B, tf, tb, slots=slots, distance=distance,
                                      n_out=Fr(1, 32)).values()) == 3302


def test_simulated_iteration_limits_and_monotonicity():
    """With a link of unbounded speed the iteration is the sum of the visits' compute times; with unbounded
    compute it is at least each direction's serial traffic and at most their sum; a faster link, more slots or
    a larger prefetch distance never make it longer."""
    rng = np.random.default_rng(5)
    spec = _toy(3)
    R = spec.n_layers
    P = [om.layer_param_count(spec, l) for l in range(R)]
    for P_B in list(all_packings(R))[::2]:
        P_F = [(0, P_B[-1][0])] if P_B[-1][0] else []
        tf = [int(x) for x in rng.integers(1, 50, R)]
        tb = [3 * x for x in tf]
        n_vis_F = sum(tf[l] for (a, e) in P_F for l in range(a, e))
        total_compute = 2 * (n_vis_F + sum(tb))
        tiny = Fr(1, 10 ** 12)
        t = _sim(spec, P_F, P_B, tf, tb, n_in=tiny, n_out=tiny)
        assert 0 <= max(e for _, e in t.values()) - total_compute < Fr(1, 1000)
        zero = [0] * R
        t = _sim(spec, P_F, P_B, zero, zero)
        n_ck = max(len(P_B) - 2, 0)
        h2d = Fr(4 * (2 * sum(P) - sum(P[P_B[-1][0]:])) + 8 * sum(P) + n_ck * 2 * 64, 64)
        d2h = Fr(16 * sum(P) + n_ck * 2 * 64, 64)
        end = max(e for _, e in t.values())
        assert max(h2d, d2h) <= end <= h2d + d2h
        prev = None
        for slots, distance in ((2, 1), (3, 1), (3, 2), (4, 3)):
            end = max(e for _, e in _sim(spec, P_F, P_B, tf, tb, slots=slots, distance=distance).values())
            assert prev is None or end <= prev
            prev = end
            assert max(e for _, e in _sim(spec, P_F, P_B, tf, tb, slots=slots, distance=distance, n_in=Fr(1, 128),
                                          n_out=Fr(1, 128)).values()) <= end
        # dropping the consumed gradient shortens the outgoing operation of every update
        assert max(e for _, e in _sim(spec, P_F, P_B, tf, tb, export_gradients=False).values()) <= \
            max(e for _, e in _sim(spec, P_F, P_B, tf, tb).values())


def test_simulated_slowdown_beside_a_busy_link_worked_by_hand():
    """The generic rule first: c takes 10 alone and 16 beside a busy `y`; `y` has work listed before c that ends at
    4, 10 or 30 while c starts at 0: backlog 4 / 10 / 30 of c's 10 -> 10 + 6 * 0.4 = 12.4, 16, 16; nothing listed: 10.
    Then the three-visit iteration of the first hand-worked test with backward times doubled beside traffic
    (C2 = 66 alone, 132 beside): when C2 starts at 195 the outgoing link holds Out1 until 415, a backlog of 220 > 66,
    so C2 takes all of 132 and ends at 327; K2 (asked at 327, link free at 305) 327-439, Out2 415-639 as before.
    C1 starts at 111 with nothing outgoing queued: 84 as alone."""
    for busy_until, want in ((4, Fr(62, 5)), (10, 16), (30, 16)):
        t = osim.run([osim.Op("w", "y", Fr(busy_until)), osim.Op("c", "x", Fr(10), stretch=("y", 16))])
        assert t["c"] == (0, want)
    assert osim.run([osim.Op("c", "x", Fr(10), stretch=("y", 16)), osim.Op("w", "y", Fr(30))])["c"] == (0, 10)
    tf, tb = [1, 10, 10, 4], [3, 30, 30, 12]
    t = _sim(_toy(2), [(0, 2)], [(0, 2), (2, 4)], tf, tb, t_fwd_beside=tf, t_bwd_beside=[2 * x for x in tb])
    assert t["C1"] == (111, 195) and t["C2"] == (195, 327) and t["K2"] == (327, 439) and t["Out2"] == (415, 639)
    # the same second set of times changes nothing; a larger one never shortens the iteration
    same = _sim(_toy(2), [(0, 2)], [(0, 2), (2, 4)], tf, tb, t_fwd_beside=tf, t_bwd_beside=tb)
    assert same == _sim(_toy(2), [(0, 2)], [(0, 2), (2, 4)], tf, tb)
    spec = _toy(4)
    P_F, P_B = [(0, 5)], [(i, i + 1) for i in range(6)]
    tf, tb = [10, 100, 100, 100, 100, 40], [30, 200, 200, 200, 200, 120]
    base = max(e for _, e in _sim(spec, P_F, P_B, tf, tb, n_out=Fr(1, 32)).values())
    prev = base
    for k in (Fr(11, 10), Fr(3, 2), 2):
        end = max(e for _, e in _sim(spec, P_F, P_B, tf, tb, n_out=Fr(1, 32), t_fwd_beside=[k * x for x in tf],
                                     t_bwd_beside=[k * x for x in tb]).values())
        assert end >= prev
        prev = end
    assert prev > base
