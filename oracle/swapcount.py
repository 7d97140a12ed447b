"""Host-link swap volumes of one iteration, as integers (bytes).

TEST INFRASTRUCTURE.  Three independent ways to the same numbers:

  closed_form()      formulas per tensor kind, following the paper's swap
                     analysis (Section 3 "Intuitive Example", and the appendix
                     "Additional Swap Analysis") specialised to one GPU;
  ledger()           walks the ordered task list (Algorithm 3) and adds what
                     each task swaps in and out;
  residency_machine  a tiny virtual-memory model: a device that can hold the
                     state of ONE pack; it executes a sequence of compute steps
                     and counts what must cross the link.  Driven in
                     microbatch-major order with write-back of everything it
                     evicts it reproduces the paper's (4m+2)|W| for the
                     per-GPU-swap baseline; driven in layer-pack-major order
                     it reproduces the paper's 3|W|.

Tensor kinds follow the paper's Figure "Tensors that need to be swapped":
W weights, dW weight gradients, K optimizer state, sX stashed pack inputs,
X/Y and dY/dX activations between packs; plus the token ids and targets.

Readings (the paper leaves these open):
  * clean weights are never written back after a forward task (the paper's
    Harmony count is in, in, out);
  * the last backward pack is shared with the forward pass (jit-compute), so
    its weights come in once, not twice: 3|W| becomes 3|W| - |W_last|;
  * the paper moves no dW at all (Section 3, second optimisation: the update
    consumes it while it is resident); an API that returns gradients exports them
    once (own kind, g_bytes per parameter) so W and K still match the paper, and
    `export_gradients=False` is the paper's own count;
  * activations between packs stay in device memory on one GPU (X/Y, dY/dX = 0);
  * pack 0's checkpoint is the token ids, and the last pack needs none, so
    max(n_B - 2, 0) checkpoints per microbatch cross the link each way.
"""
from __future__ import annotations

from . import model as om
from . import schedule as osch

KINDS = ("W", "dW", "K", "sX", "XY", "dXdY", "ids")


def bytes_per_param(precision: str):
    """(w_c, k_B, g_B): compute-precision weight, optimizer state, exported grad.
    'fp32': the fp32 weight is the master; K = (m, v).
    'bf16': bf16 weight + K = (fp32 master, m, v)."""
    if precision == "fp32":
        return 4, 8, 4
    if precision == "bf16":
        return 2, 12, 4
    raise ValueError(precision)


def _pcount(spec, a, e):
    return sum(om.layer_param_count(spec, l) for l in range(a, e))


def closed_form(spec: om.Spec, P_F, P_B, M: int, b: int, precision: str, update_on_host: bool = False,
                export_gradients: bool = True, resident_K_params: int = 0, resident_K_loaded: bool = True,
                M_F: int | None = None, b_F: int | None = None):
    """Layer-pack-major volumes.  Returns {'h2d': {kind: bytes}, 'd2h': {...}}.

    M, b: the backward pass's microbatches (M_B of U_B sequences).  M_F, b_F: the forward
    pass's (M_F of U_F), if the configuration uses distinct sizes (Section 4.3.1); the
    checkpoints then go out once per forward microbatch in its size and come back once per
    backward microbatch in that one's -- the same bytes, since both cover the minibatch.

    resident_K_params: parameters whose optimizer state is pinned on the device
    (Algorithm 3 lists a channel that keeps a tensor on the GPU beside the CPU-GPU
    swap): their K crosses the link neither way, except once, inwards, in the first
    iteration after the host arrays were handed over (resident_K_loaded=False).
    Their weights and gradients move like everybody else's.

    export_gradients=False: the update on the device drops the gradient it has
    consumed, as in the paper, where dW never moves (no effect with update_on_host,
    where the gradient is what the CPU reads).

    update_on_host: the Weight Update task runs on the CPU (Section 4.4, first
    paragraph: the Runtime supports offloading it).  The optimizer state and the
    updated weights then never cross the link: the host reads the gradient that the
    backward task exported and writes W and K where they already live."""
    osch.check_packs(spec, P_F, P_B)
    w_c, k_B, g_B = bytes_per_param(precision)
    P_all = _pcount(spec, 0, spec.n_layers)
    P_last = _pcount(spec, *P_B[-1])
    T = b * spec.seq_len
    a = T * spec.d_model * w_c
    n_ckpt = max(len(P_B) - 2, 0)
    h2d = dict.fromkeys(KINDS, 0)
    d2h = dict.fromkeys(KINDS, 0)
    h2d["W"] = w_c * (2 * P_all - P_last)
    d2h["W"] = w_c * P_all
    d2h["dW"] = g_B * P_all
    h2d["K"] = k_B * P_all
    d2h["K"] = k_B * P_all
    h2d["sX"] = M * a * n_ckpt
    if M_F is None and b_F is None:
        M_F, b_F = M, b
    if M_F * b_F != M * b:
        raise ValueError("both passes must cover the same minibatch")
    d2h["sX"] = M_F * (b_F * spec.seq_len * spec.d_model * w_c) * n_ckpt
    h2d["ids"] = 2 * M * T * 4
    if update_on_host:
        h2d["K"] = d2h["K"] = d2h["W"] = 0
    else:
        if not 0 <= resident_K_params <= P_all:
            raise ValueError("resident_K_params")
        d2h["K"] -= k_B * resident_K_params
        if resident_K_loaded:
            h2d["K"] -= k_B * resident_K_params
        if not export_gradients:
            d2h["dW"] = 0
    return {"h2d": h2d, "d2h": d2h}


def closed_form_microbatch_major(spec: om.Spec, P_F, P_B, M: int, b: int, precision: str,
                                 update_on_host: bool = False, export_gradients: bool = True,
                                 resident_K_params: int = 0, resident_K_loaded: bool = True):
    """Same packs, same one-pack-at-a-time residency, but every microbatch runs
    through all packs before the next one starts (the per-GPU-swap order of
    Section 3, "Intuitive Example").  Weights come in M times.  A pack's gradient
    buffer cannot stay on the device between microbatches either (appendix
    "Additional Swap Analysis": dW swaps like W, in the backward pass only): it
    goes out after every backward task and comes back in before the next
    microbatch's.  Readings: the first microbatch starts from a zero-filled buffer
    (nothing to bring in); the last microbatch's gradient is consumed on the device
    by the update that follows it and leaves once, as the exported gradient -- so
    M - 1 times in and M times out (M - 1 out when a device update drops it instead
    of exporting it), against the paper's 2m + 2 for a system that also swaps around
    a separate update phase."""
    out = closed_form(spec, P_F, P_B, M, b, precision, update_on_host, export_gradients, resident_K_params,
                      resident_K_loaded)
    w_c, k_B, g_B = bytes_per_param(precision)
    P_all = _pcount(spec, 0, spec.n_layers)
    out["h2d"]["W"] *= M
    out["h2d"]["dW"] = (M - 1) * g_B * P_all
    out["d2h"]["dW"] += (M - 1) * g_B * P_all
    return out


def update_chunks(spec: om.Spec, P_B, chunk_params: int):
    """The pieces in which the update tasks handle optimizer state, in the order the
    iteration reaches them: backward packs in reverse (Algorithm 3), each pack's
    parameters in storage order in runs of chunk_params.  Returns a list of
    (pack, index within the pack, parameters)."""
    out = []
    for pack in reversed(P_B):
        n = _pcount(spec, *pack)
        for c in range(-(-n // chunk_params)):
            out.append((pack, c, min(chunk_params, n - c * chunk_params)))
    return out


def ledger(spec: om.Spec, P_F, P_B, M: int, b: int, precision: str, update_on_host: bool = False,
           export_gradients: bool = True, chunk_params: int | None = None, resident=frozenset(),
           resident_loaded: bool = True, M_F: int | None = None, b_F: int | None = None):
    """Add up what every task of the ordered list swaps.  M, b are the backward pass's
    microbatches; forward tasks run M_F microbatches of b_F sequences (default: the same).

    resident: set of (pack, index) from update_chunks(spec, P_B, chunk_params) whose
    optimizer state is pinned on the device (Algorithm 3 lists such a channel beside the
    CPU-GPU swap): an update task moves that piece's state neither way, except inwards
    once, at its first update after the host arrays were handed over
    (resident_loaded=False).  Weights and gradients of the piece move as always."""
    if resident and chunk_params is None:
        raise ValueError("resident pieces need chunk_params")
    w_c, k_B, g_B = bytes_per_param(precision)
    T = b * spec.seq_len
    act = T * spec.d_model * w_c
    h2d = dict.fromkeys(KINDS, 0)
    d2h = dict.fromkeys(KINDS, 0)
    h2d["ids"] += M * T * 4       # token ids
    h2d["ids"] += M * T * 4       # targets
    if M_F is None and b_F is None:
        M_F, b_F = M, b
    act_F = b_F * spec.seq_len * spec.d_model * w_c
    for t in osch.task_list(spec, P_F, P_B):
        npar = _pcount(spec, *t.pack)
        if t.kind == "F":
            h2d["W"] += w_c * npar
            for _layer in t.stash_out_layers:
                for _mb in range(M_F):
                    d2h["sX"] += act_F
        elif t.kind == "B":
            h2d["W"] += w_c * npar
            if t.stash_in_layer is not None:
                for _mb in range(M):
                    h2d["sX"] += act
        elif update_on_host:
            d2h["dW"] += g_B * npar       # all the CPU needs from the device
        else:
            pieces = [(t.pack, 0, npar)] if chunk_params is None else \
                [p for p in update_chunks(spec, [t.pack], chunk_params)]
            for (pack, c, n) in pieces:
                if (pack, c) in resident:
                    if not resident_loaded:
                        h2d["K"] += k_B * n
                else:
                    h2d["K"] += k_B * n
                    d2h["K"] += k_B * n
                d2h["W"] += w_c * n
                if export_gradients:
                    d2h["dW"] += g_B * n
    return {"h2d": h2d, "d2h": d2h}


def ledger_microbatch_major(spec: om.Spec, P_F, P_B, M: int, b: int, precision: str, update_on_host: bool = False,
                            export_gradients: bool = True):
    """Add up what every task of the microbatch-major list swaps."""
    w_c, k_B, g_B = bytes_per_param(precision)
    T = b * spec.seq_len
    act = T * spec.d_model * w_c
    h2d = dict.fromkeys(KINDS, 0)
    d2h = dict.fromkeys(KINDS, 0)
    h2d["ids"] += M * T * 4       # token ids
    h2d["ids"] += M * T * 4       # targets
    has_gradient = set()          # packs whose buffer holds earlier microbatches' sums
    for t in osch.task_list_microbatch_major(spec, P_F, P_B, M):
        npar = _pcount(spec, *t.pack)
        if t.kind == "F":
            h2d["W"] += w_c * npar
            d2h["sX"] += act * len(t.stash_out_layers)
        elif t.kind == "B":
            h2d["W"] += w_c * npar
            if t.stash_in_layer is not None:
                h2d["sX"] += act
            if t.pack in has_gradient:
                h2d["dW"] += g_B * npar
            has_gradient.add(t.pack)
            if t.mb != M - 1:                 # else the update that follows takes it from the device
                d2h["dW"] += g_B * npar
        elif update_on_host:
            d2h["dW"] += g_B * npar
        else:
            h2d["K"] += k_B * npar
            d2h["K"] += k_B * npar
            d2h["W"] += w_c * npar
            if export_gradients:
                d2h["dW"] += g_B * npar
    return {"h2d": h2d, "d2h": d2h}


# --------------------------------------------------------------------------
# the paper's own formulas (Section 3, "Intuitive Example")
# --------------------------------------------------------------------------

def paper_W_volume_per_gpu_swap_dp(m: int, N: int, W: int) -> int:
    """Data parallelism with per-GPU memory virtualisation: (4m + 2) N |W|."""
    return (4 * m + 2) * N * W


def paper_W_volume_harmony_dp(N: int, W: int) -> int:
    """Harmony DP: in once for forward, in once for backward, out once: 3 N |W|."""
    return 3 * N * W


def paper_dW_volume_per_gpu_swap_dp(m: int, N: int, W: int) -> int:
    """Appendix: like W but with 2m deducted (no dW in the forward pass)."""
    return (2 * m + 2) * N * W


def paper_K_volume(N: int, K: int) -> int:
    """Appendix: optimizer state in and out once per GPU in the update phase."""
    return 2 * N * K


# --------------------------------------------------------------------------
# residency machine: an independent count from first principles
# --------------------------------------------------------------------------

def residency_machine(steps, pack_bytes, write_back_clean: bool):
    """A device holding the weights of at most one pack.

    steps: sequence of (pack_id, writes) in execution order; `writes` says the
    step leaves the pack's weights modified (the update).  Before a step runs,
    its pack must be resident: whatever else is resident is evicted (written
    back if dirty, or always if `write_back_clean` -- a virtual-memory system
    that does not track cleanliness swaps out all it evicts), then the pack is
    read in.  At the end the resident pack is evicted the same way.
    Returns (bytes_in, bytes_out)."""
    resident, dirty = None, False
    b_in = b_out = 0

    def evict():
        nonlocal resident, dirty, b_out
        if resident is not None and (dirty or write_back_clean):
            b_out += pack_bytes[resident]
        resident, dirty = None, False

    for pack_id, writes in steps:
        if pack_id is None:          # end of a pass: nothing stays resident
            evict()
            continue
        if resident != pack_id:
            evict()
            b_in += pack_bytes[pack_id]
            resident = pack_id
        dirty = dirty or writes
    evict()
    return b_in, b_out


FLUSH = (None, False)


def steps_microbatch_major(n_packs: int, M: int, independent_passes: bool):
    """Per-GPU-swap baseline: per microbatch all packs forward then all packs
    backward; the update of every pack only after the whole backward pass.
    `independent_passes` is the paper's simplification that every pass starts
    with nothing resident (it ignores the pack that happens to be shared at
    each turnaround)."""
    steps = []
    for _mb in range(M):
        steps += [(p, False) for p in range(n_packs)]
        if independent_passes:
            steps.append(FLUSH)
        steps += [(p, False) for p in reversed(range(n_packs))]
        if independent_passes:
            steps.append(FLUSH)
    steps += [(p, True) for p in range(n_packs)]
    return steps


def steps_layer_pack_major(n_packs: int, M: int, share_last: bool):
    """Harmony: each pack forward over all microbatches, then each pack backward
    over all microbatches followed at once by its update (jit-update, while the
    pack is still resident).  With `share_last` the last pack's forward and
    backward are one visit (jit-compute); without it the two passes are
    independent, as in the paper's simplified count."""
    steps = []
    n_fwd = n_packs - 1 if share_last else n_packs
    for p in range(n_fwd):
        steps += [(p, False)] * M
    if not share_last:
        steps.append(FLUSH)
    for p in reversed(range(n_packs)):
        steps += [(p, False)] * M
        steps += [(p, True)]
    return steps
