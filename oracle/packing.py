"""Balanced-time packing (the paper's Algorithm 2) written out step by step.

TEST INFRASTRUCTURE.  Given per-layer times t and per-layer memory footprints m
for one pass type and one microbatch size, and the memory capacity alpha, try
S = S_min, S_min+1, ... packs: aim at equal per-pack time by cutting the prefix
sum of t at c, 2c, ..., (S-1)c with c = sum(t)/S, and return the first S whose
every pack fits alpha.  For forward packing the last backward pack is removed
first (jit-compute), so P_F covers only the layers before it.

Readings where the listing is silent:
  * S_min = ceil(sum(m)/alpha), at least 1;
  * the cut for target k*c is the number of layers whose prefix time is
    <= k*c ("insert to the right"), evaluated in integers as
    prefix*S <= k*sum(t) so that ties are exact: four equal layers in two
    packs split 2+2;
  * a cut that repeats the previous one (a single layer longer than c) or
    falls at 0 yields no pack (empty packs are dropped);
  * a pack over capacity means "try S+1"; with unequal times even S = R need
    not separate all layers, so if the loop ends without a feasible split the
    packing falls back to one layer per pack, and only if that does not fit
    either is there no packing (None);
  * `also_fits`, if given, is a further whole-packing feasibility test ANDed
    to the per-pack test (the runtime's arena must hold the largest pack state
    twice plus the largest pack's activations, which can come from different
    packs).
Times and memories are integers (analytic flop and byte counts).

Parity unpinned: the exact pack boundaries of the paper's table of layer packs
(they come from its measured layer times).  Pinned instead: properties, brute
force on small cases, and the structure of that table (pack counts per size).
"""
from __future__ import annotations


def split_points(t, S: int):
    """Layer counts i_1 <= ... <= i_{S-1}: i_k = #{j : prefix_j * S <= k * total}."""
    total = sum(t)
    prefix = []
    acc = 0
    for x in t:
        acc += x
        prefix.append(acc)
    cuts = []
    for k in range(1, S):
        cuts.append(sum(1 for p in prefix if p * S <= k * total))
    return cuts


def packs_from_cuts(cuts, R: int, first: int = 0):
    bounds = [0] + list(cuts) + [R]
    packs = []
    for a, e in zip(bounds[:-1], bounds[1:]):
        if e > a:
            packs.append((first + a, first + e))
    return packs


def balanced_time_packing(t, m, alpha: int, also_fits=None, first: int = 0, S_start: int = 1, with_S: bool = False):
    """Algorithm 2 on explicit lists.  Returns a list of (start, end) packs over
    layers first..first+len(t), or None if no S <= R fits.  The loop starts at
    max(S_min, S_start); with_S also returns the accepted pack count (R + 1 for the
    one-layer-per-pack fallback), so a caller can enumerate further candidates."""
    R = len(t)
    assert len(m) == R

    def ret(packs, S):
        return (packs, S) if with_S else packs
    if R == 0:
        return ret([], 0)
    if alpha <= 0:
        return ret(None, 0)
    S_min = max(1, -(-sum(m) // alpha))
    for S in range(max(S_min, S_start), R + 1):
        packs = packs_from_cuts(split_points(t, S), R, first)
        ok = all(sum(m[a - first:e - first]) <= alpha for (a, e) in packs)
        if ok and also_fits is not None:
            ok = also_fits(packs)
        if ok:
            return ret(packs, S)
    if S_start > R + 1:
        return ret(None, 0)
    packs = [(first + j, first + j + 1) for j in range(R)]
    if all(mj <= alpha for mj in m) and (also_fits is None or also_fits(packs)):
        return ret(packs, R + 1)
    return ret(None, 0)


def forward_layers_given_backward(P_B):
    """Number of layers the forward packing covers: all before P_B's last pack."""
    return P_B[-1][0]


# --------------------------------------------------------------------------
# analytic layer profile and device-memory model of the runtime under test
# --------------------------------------------------------------------------
# The paper's Profiler measures per-layer time, memory and activation size
# (Section 4.2).  Here they are computed: "time" is the flop count of one
# microbatch; memory follows the runtime's arena, written out below from its
# description (N_SLOTS weight slots -- the pack in use, the next one arriving, the
# previous one draining through its update --, one activation workspace, a
# pack-independent reserve), every buffer rounded up to 256 bytes.

def _a256(x: int) -> int:
    return (x + 255) // 256 * 256


N_SLOTS = 3
OUT_RING, IN_RING, K_RING = 4, 4, 3
K_CHUNK_MAX = 4 * 2 ** 20
LOGIT_ROWS = 512
LN_BLOCKS = 256


def elem_bytes(precision: str) -> int:
    return {"fp32": 4, "bf16": 2}[precision]


def block_act_bytes(spec, b: int, precision: str) -> int:
    """What one microbatch keeps per block for backward: x_in, LN1 out, qkv,
    attention out, x_mid, LN2 out, MLP pre- and post-activation, two LayerNorm
    (mean, rstd) pairs and the attention logsumexp."""
    E = elem_bytes(precision)
    T, d, f, H = b * spec.seq_len, spec.d_model, spec.d_ffn, spec.n_heads
    sizes = [T * d * E, T * d * E, 3 * T * d * E, T * d * E, T * d * E, T * d * E, T * f * E, T * f * E,
             T * 4, T * 4, T * 4, T * 4, T * H * 4]
    return sum(_a256(x) for x in sizes)


def head_act_bytes(spec, b: int, precision: str) -> int:
    """Head input, final-LN output, its (mean, rstd), one chunk of logits (fp32),
    their gradient for the whole microbatch (element type; rows padded to a
    multiple of 64 elements), plus an fp32 [T, d] accumulator for the gradient of the LN output."""
    E = elem_bytes(precision)
    T, d = b * spec.seq_len, spec.d_model
    rows = min(T, LOGIT_ROWS)
    ldl = (spec.vocab + 63) // 64 * 64
    sizes = [T * d * E, T * d * E, T * 4, T * 4, rows * ldl * 4, T * ldl * E, T * d * 4]
    return sum(_a256(x) for x in sizes)


def layer_profile(spec, M: int, b: int, precision: str):
    """Per layer: dict(t_fwd, t_bwd, params, mem_fwd, mem_bwd, act_bwd)."""
    from . import model as om
    E = elem_bytes(precision)
    T, d, f, V, s = b * spec.seq_len, spec.d_model, spec.d_ffn, spec.vocab, spec.seq_len
    out = []
    for layer in range(spec.n_layers):
        p = om.layer_param_count(spec, layer)
        if layer == 0:
            t_f, act = T * d, 0
        elif layer <= spec.n_blocks:
            t_f = T * (8 * d * d + 4 * d * f + (2 if spec.causal else 4) * s * d)
            act = block_act_bytes(spec, b, precision)
        else:
            t_f, act = 2 * T * d * V, head_act_bytes(spec, b, precision)
        out.append(dict(t_fwd=t_f, t_bwd=3 * t_f, params=p, mem_fwd=N_SLOTS * E * p,
                        mem_bwd=N_SLOTS * (E + 4) * p + act, act_bwd=act))
    return out


def reserved_bytes(spec, M: int, b: int, precision: str) -> int:
    """Pack-independent device memory: resident boundary activations (one per
    microbatch), pack-input ring, checkpoint staging ring, gradient scratch,
    ids and targets, a 4 KiB scalar page, the LayerNorm-backward partial sums
    (LN_BLOCKS rows of 2 d floats) and the optimizer-state ring."""
    from . import model as om
    E = elem_bytes(precision)
    T, d, f, H = b * spec.seq_len, spec.d_model, spec.d_ffn, spec.n_heads
    x = _a256(T * d * E)
    total = _a256(M * x) + _a256(IN_RING * x) + _a256(OUT_RING * x)
    total += _a256(T * max(f, 3 * d) * E) + _a256(T * d * E) + _a256(T * H * 4)
    total += 2 * _a256(M * T * 4) + 4096 + _a256(LN_BLOCKS * 2 * d * 4)
    chunk = min(K_CHUNK_MAX, max(om.layer_param_count(spec, l) for l in range(spec.n_layers)))
    n_k = 3 if precision == "bf16" else 2
    total += _a256(K_RING * n_k * _a256(chunk * 4))
    return total


def arena_bytes(spec, P_F, P_B, M: int, b: int, precision: str):
    """(total, slot_bytes, act_bytes): reserve + N_SLOTS weight slots + the largest
    backward pack's activation workspace."""
    from . import model as om
    E = elem_bytes(precision)
    prof = layer_profile(spec, M, b, precision)

    def npar(a, e):
        return sum(om.layer_param_count(spec, l) for l in range(a, e))
    slot = 0
    for (a, e) in P_F:
        slot = max(slot, _a256(E * npar(a, e)))
    act = 0
    for (a, e) in P_B:
        slot = max(slot, _a256(E * npar(a, e)) + _a256(4 * npar(a, e)))
        act = max(act, sum(prof[l]["act_bwd"] for l in range(a, e)))
    return reserved_bytes(spec, M, b, precision) + N_SLOTS * slot + act, slot, act


HOST_PARAMS_PER_NS = 6      # CPU update threads: about 6 parameters per nanosecond


def estimate_iteration_ns(spec, P_F, P_B, M: int, b: int, precision: str, link_MBps: int, compute_GFLOPs: int,
                          update_on_host: bool = False) -> int:
    """Runtime estimate of one iteration (the role of the paper's Runtime Estimator,
    reduced to one GPU): an event-driven walk of the task list over the compute
    stream and the two directions of the host link, in integer nanoseconds.
    A visit computes for n_micro * (sum of its layers' flops) / rate; its weights
    are requested when the previous visit starts computing and its slot (visit
    index mod 2) is free; a backward visit's update moves the optimizer state in and
    (state + weights + fp32 gradients) out after its compute ends; the two links
    are each one queue.  Checkpoint traffic is ignored.  update_on_host: nothing comes
    in for the update, only the fp32 gradient goes out, and the CPU threads are one
    more queue (Section 4.4: the update task placed on the CPU)."""
    from . import model as om
    E = elem_bytes(precision)
    kB = 12 if precision == "bf16" else 8
    prof = layer_profile(spec, M, b, precision)

    def t_bytes(n):
        return -(-n * 1000 // link_MBps)

    def t_flops(n):
        return -(-n // compute_GFLOPs)

    def npar(a, e):
        return sum(om.layer_param_count(spec, l) for l in range(a, e))
    visits = []
    for (a, e) in P_F:
        visits.append((False, t_flops(M * sum(prof[l]["t_fwd"] for l in range(a, e))), t_bytes(E * npar(a, e)), 0, 0, 0))
    for (a, e) in reversed(P_B):
        P = npar(a, e)
        comp = t_flops(M * sum(prof[l]["t_bwd"] for l in range(a, e)))
        if update_on_host:
            visits.append((True, comp, t_bytes(E * P), 0, t_bytes(4 * P), P // HOST_PARAMS_PER_NS))
        else:
            visits.append((True, comp, t_bytes(E * P), t_bytes(kB * P), t_bytes((kB + E + 4) * P), 0))
    h2d_free = d2h_free = comp_free = cpu_free = 0
    slot_free = [0] * N_SLOTS
    w_ready = [0] * (len(visits) + 1)
    w_ready[0] = visits[0][2]
    h2d_free = w_ready[0]
    for v, (bwd, comp, w, kin, out, cpu) in enumerate(visits):
        comp_start = max(comp_free, w_ready[v])
        if v + 1 < len(visits):
            s = max(comp_start, slot_free[(v + 1) % N_SLOTS], h2d_free)
            w_ready[v + 1] = s + visits[v + 1][2]
            h2d_free = w_ready[v + 1]
        comp_end = comp_start + comp
        comp_free = comp_end
        if not bwd:
            slot_free[v % N_SLOTS] = comp_end
        else:
            kin_end = comp_end
            if not update_on_host:
                kin_end = max(comp_end, h2d_free) + kin
                h2d_free = kin_end
            out_end = max(max(comp_end, d2h_free) + out, kin_end)
            d2h_free = out_end
            slot_free[v % N_SLOTS] = out_end
            if update_on_host:
                cpu_free = max(cpu_free, out_end) + cpu
    return max(comp_free, d2h_free, cpu_free)


def taper_first_pack(P_B):
    """[0, e) -> [0,1), [1,2), [2,e): the pack visited last gets the smallest update."""
    e = P_B[0][1]
    if e < 2:
        return list(P_B)
    head = [(0, 1), (1, 2)] + ([(2, e)] if e > 2 else [])
    return head + list(P_B[1:])


def merge_last_packs(P_B):
    """The last two backward packs become one (less recompute, shorter forward pass)."""
    if len(P_B) < 2:
        return list(P_B)
    return list(P_B[:-2]) + [(P_B[-2][0], P_B[-1][1])]


def plan(spec, budget: int, M: int, b: int, precision: str, search: int = 0, link_MBps: int = 40000,
         compute_GFLOPs: int = 420000, update_on_host: bool = False):
    """Backward packs by Algorithm 2 on (t_bwd, mem_bwd) with capacity budget -
    reserve and the whole-arena test; then forward packs on (t_fwd, mem_fwd)
    over the layers before the last backward pack with capacity N_SLOTS * slot.
    search = 0 keeps the first feasible pack count (Algorithm 2 alone); search = n
    also tries the next n feasible pack counts, each also with its first pack
    tapered, its last two packs merged, and both (where the arena still fits), each with
    balanced forward packs and with forward packs doubling in size from two layers, and,
    as Algorithm 1 does over its configurations, keeps the candidate with the
    smallest estimated iteration time (ties: the earlier one).  Returns (P_F, P_B)
    or None."""
    prof = layer_profile(spec, M, b, precision)
    res = reserved_bytes(spec, M, b, precision)
    if budget <= res:
        return None
    fits = lambda packs: arena_bytes(spec, [], packs, M, b, precision)[0] <= budget
    state = dict(best=None, ns=None, failed=False)

    def consider(P_B):
        slot = arena_bytes(spec, [], P_B, M, b, precision)[1]
        RF = forward_layers_given_backward(P_B)
        P_F = balanced_time_packing([p["t_fwd"] for p in prof[:RF]], [p["mem_fwd"] for p in prof[:RF]], N_SLOTS * slot)
        if P_F is None:
            state["failed"] = True
            return
        def offer(P_F):
            ns = estimate_iteration_ns(spec, P_F, P_B, M, b, precision, link_MBps, compute_GFLOPs, update_on_host)
            if state["best"] is None or ns < state["ns"]:
                state["best"], state["ns"] = (P_F, P_B), ns

        offer(P_F)
        if search > 0 and RF > 2:
            # forward packs that double in size from two layers on: the first pack's
            # load is the part of the forward pass nothing can hide
            G, a, size, ok = [], 0, 2, True
            while a < RF:
                e = min(RF, a + size)
                if RF - e < size:
                    e = RF
                if sum(p["mem_fwd"] for p in prof[a:e]) > N_SLOTS * slot:
                    ok = False
                G.append((a, e))
                a, size = e, size * 2
            if ok:
                offer(G)

    S_start = 1
    for _ in range(search + 1):
        P_B, S_used = balanced_time_packing(
            [p["t_bwd"] for p in prof], [p["mem_bwd"] for p in prof], budget - res,
            also_fits=fits, S_start=S_start, with_S=True)
        if P_B is None:
            break
        consider(P_B)
        if search > 0:
            t = taper_first_pack(P_B)
            if len(t) != len(P_B) and fits(t):
                consider(t)
            if len(P_B) >= 2:
                g = merge_last_packs(P_B)
                if fits(g):
                    consider(g)
                    tg = taper_first_pack(g)
                    if len(tg) != len(g) and fits(tg):
                        consider(tg)
        if state["failed"]:
            return None
        if S_used > spec.n_layers:
            break
        S_start = S_used + 1
    return state["best"]
