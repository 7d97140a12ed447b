"""The layer-pack-major iteration of the paper, driven over the oracle's layers.

TEST INFRASTRUCTURE.  The same per-layer functions as `model.py`, executed in
the order the paper's Runtime executes them on one GPU (Section 3, "Key
Optimizations"; Section 4.3.2 and Algorithm 3 for the task order):

  * input-batch grouping: a forward task runs its layer pack over ALL
    microbatches before the next pack starts;
  * the forward pass keeps only the INPUT of each backward pack (the
    checkpoint, Section 4.3.1 first bullet); a backward task first recomputes
    the pack's forward from that input, then runs its backward;
  * jit-compute: the last backward pack is shared with the forward pass and
    runs forward+backward per microbatch, with no recompute;
  * jit-update: the optimizer step of a pack directly follows its backward task.

Because the result must equal ordinary synchronous training exactly, this
driver is also a pin on the oracle: its gradients must be bit-identical to
`iteration_microbatch_major` (each tensor still receives its microbatch
contributions in ascending order; only the interleaving across layers differs).

Packs are lists of (first_layer, end_layer) half-open ranges over the R layers.
P_B covers 0..R; P_F covers exactly the layers before P_B's last pack
(Algorithm 2, first two lines).
"""
from __future__ import annotations

from dataclasses import dataclass, field

from . import model as om


def check_packs(spec: om.Spec, P_F, P_B) -> None:
    R = spec.n_layers
    if not P_B:
        raise ValueError("P_B is empty")
    pos = 0
    for (a, e) in P_B:
        if a != pos or e <= a:
            raise ValueError(f"P_B not contiguous/non-empty at {(a, e)}")
        pos = e
    if pos != R:
        raise ValueError("P_B does not cover all layers")
    last_start = P_B[-1][0]
    pos = 0
    for (a, e) in P_F:
        if a != pos or e <= a:
            raise ValueError(f"P_F not contiguous/non-empty at {(a, e)}")
        pos = e
    if pos != last_start:
        raise ValueError("P_F must cover exactly the layers before P_B's last pack")


@dataclass
class Task:
    """One entry of the ordered task list (Algorithm 3 at N = 1).
    kind: 'F' forward, 'B' backward (recompute + backward, or forward +
    backward for the last pack), 'A' update."""
    index: int
    kind: str
    pack: tuple
    is_last_pack: bool = False
    stash_out_layers: list = field(default_factory=list)  # F: inputs checkpointed
    stash_in_layer: int | None = None                      # B: checkpoint consumed
    mb: int | None = None    # None: the task runs every microbatch (input-batch grouping); else this one


def task_list(spec: om.Spec, P_F, P_B):
    """Forward tasks in pack order, then (backward, update) pairs in reverse
    pack order (Algorithm 3, the two creation loops)."""
    check_packs(spec, P_F, P_B)
    ckpt_layers = {a for (a, _) in P_B[1:-1]}   # inputs that must be stashed
    tasks = []
    for pack in P_F:
        t = Task(len(tasks), "F", pack)
        t.stash_out_layers = [l for l in range(pack[0], pack[1]) if l in ckpt_layers]
        tasks.append(t)
    for k in reversed(range(len(P_B))):
        pack = P_B[k]
        last = (k == len(P_B) - 1)
        t = Task(len(tasks), "B", pack, is_last_pack=last)
        if not last and pack[0] != 0:
            t.stash_in_layer = pack[0]
        tasks.append(t)
        tasks.append(Task(len(tasks), "A", pack, is_last_pack=last))
    return tasks


def task_list_microbatch_major(spec: om.Spec, P_F, P_B, M: int):
    """The order the paper compares against (Section 3, "Intuitive Example": memory
    virtualisation per GPU, every microbatch on its own), over the SAME packs: for each
    microbatch all forward packs, then all backward packs in reverse.  Nothing is grouped,
    so every task names its microbatch.  The update of a pack still follows the backward
    task that completes its gradient (the one of the last microbatch)."""
    tasks = []
    for mb in range(M):
        for t in task_list(spec, P_F, P_B):
            if t.kind == "A" and mb != M - 1:
                continue
            t.index = len(tasks)
            t.mb = mb
            tasks.append(t)
    return tasks


def regroup(parts, rows_per_part: int):
    """Row blocks of one minibatch cut into pieces of another size: the rows of all
    `parts` in order, re-split into blocks of rows_per_part rows."""
    import numpy as np
    rows = np.concatenate(parts, axis=0)
    assert rows.shape[0] % rows_per_part == 0
    return [rows[i:i + rows_per_part].copy() for i in range(0, rows.shape[0], rows_per_part)]


def iteration_layer_pack_major(spec: om.Spec, params, ids, targets, P_F, P_B,
                               m, v, hp: om.AdamHP, order: str = "layer_pack_major", U_F: int | None = None):
    """One iteration in task-list order.  Returns dict(loss, grads, weights, m, v).
    order = "microbatch_major" executes task_list_microbatch_major instead.

    U_F: forward microbatch size of the configuration 4-tuple (Section 4.3.1; Algorithm 1
    searches U_F and U_B separately).  ids is [M_B, U_B, s]: the backward tasks, and the
    last pack that is shared with them, run its microbatches as given; with U_F set, the
    forward tasks run the same M_B * U_B sequences in microbatches of U_F sequences, and
    the activations and checkpoints they leave are re-cut into the backward microbatches
    (every row belongs to one sequence, so only the grouping changes).  Gradients are
    summed over the backward microbatches in ascending order, as in the definition."""
    M = ids.shape[0]
    n_tgt = om.count_targets(targets)
    if U_F is not None and U_F != ids.shape[1]:
        if order != "layer_pack_major":
            raise ValueError("distinct forward and backward microbatch sizes need the layer-pack-major order")
        return _iteration_distinct_fb(spec, params, ids, targets, P_F, P_B, m, v, hp, U_F, n_tgt)
    if order == "layer_pack_major":
        tasks = task_list(spec, P_F, P_B)
    elif order == "microbatch_major":
        tasks = task_list_microbatch_major(spec, P_F, P_B, M)
    else:
        raise ValueError(order)
    X = [None] * M                    # boundary activation of each microbatch
    stash = {}                        # (layer, mb) -> checkpointed input
    grads: dict = {}
    loss = 0.0
    new_w, new_m, new_v = {}, {}, {}

    for t in tasks:
        a, e = t.pack
        mbs = range(M) if t.mb is None else (t.mb,)
        if t.kind == "F":
            for mb in mbs:
                x = X[mb]
                for layer in range(a, e):
                    if layer in t.stash_out_layers:
                        stash[(layer, mb)] = x.copy()
                    x, _ = om.layer_fwd(layer, x, params, spec, ids[mb], targets[mb], n_tgt)
                X[mb] = x
        elif t.kind == "B":
            for mb in mbs:
                b = ids[mb].shape[0]
                if a == 0:
                    x = None                  # the embedding restarts from the ids
                elif t.is_last_pack:
                    x = X[mb]                 # still resident from the forward pass
                else:
                    x = stash.pop((t.stash_in_layer, mb))
                caches = {}
                for layer in range(a, e):
                    x, caches[layer] = om.layer_fwd(layer, x, params, spec,
                                                    ids[mb], targets[mb], n_tgt)
                if t.is_last_pack:
                    loss += x
                    dy = None
                else:
                    dy = X[mb]
                for layer in reversed(range(a, e)):
                    dy, g = om.layer_bwd(layer, dy, caches[layer], params, spec, b)
                    om.accumulate(grads, g)
                X[mb] = dy               # gradient w.r.t. the pack's input
        else:  # 'A': jit-update of this pack's tensors
            for layer in range(a, e):
                for name in om.layer_param_shapes(spec, layer):
                    new_w[name], new_m[name], new_v[name] = om.adam_update(
                        params[name], grads[name], m[name], v[name], hp)
    assert not stash, "every checkpoint must be consumed exactly once"
    return {"loss": float(loss), "grads": grads, "weights": new_w, "m": new_m, "v": new_v}


def _iteration_distinct_fb(spec: om.Spec, params, ids, targets, P_F, P_B, m, v, hp: om.AdamHP, U_F: int, n_tgt: int):
    M_B, U_B, s = ids.shape
    D = M_B * U_B
    if D % U_F:
        raise ValueError("U_F must divide the minibatch")
    M_F = D // U_F
    ids_F = ids.reshape(M_F, U_F, s)
    tg_F = targets.reshape(M_F, U_F, s)
    tasks = task_list(spec, P_F, P_B)
    X_F = [None] * M_F
    stash_F = {}                      # layer -> list over forward microbatches
    for t in tasks:
        if t.kind != "F":
            continue
        a, e = t.pack
        for mb in range(M_F):
            x = X_F[mb]
            for layer in range(a, e):
                if layer in t.stash_out_layers:
                    stash_F.setdefault(layer, [None] * M_F)[mb] = x.copy()
                x, _ = om.layer_fwd(layer, x, params, spec, ids_F[mb], tg_F[mb], n_tgt)
            X_F[mb] = x
    # the hand-over between the passes: same rows, cut into the backward microbatches
    X = regroup(X_F, U_B * s) if P_F else [None] * M_B
    stash = {(layer, mb): x for layer, parts in stash_F.items() for mb, x in enumerate(regroup(parts, U_B * s))}
    grads: dict = {}
    loss = 0.0
    new_w, new_m, new_v = {}, {}, {}
    for t in tasks:
        a, e = t.pack
        if t.kind == "B":
            for mb in range(M_B):
                if a == 0:
                    x = None
                elif t.is_last_pack:
                    x = X[mb]
                else:
                    x = stash.pop((t.stash_in_layer, mb))
                caches = {}
                for layer in range(a, e):
                    x, caches[layer] = om.layer_fwd(layer, x, params, spec, ids[mb], targets[mb], n_tgt)
                if t.is_last_pack:
                    loss += x
                    dy = None
                else:
                    dy = X[mb]
                for layer in reversed(range(a, e)):
                    dy, g = om.layer_bwd(layer, dy, caches[layer], params, spec, U_B)
                    om.accumulate(grads, g)
                X[mb] = dy
        elif t.kind == "A":
            for layer in range(a, e):
                for name in om.layer_param_shapes(spec, layer):
                    new_w[name], new_m[name], new_v[name] = om.adam_update(
                        params[name], grads[name], m[name], v[name], hp)
    assert not stash, "every checkpoint must be consumed exactly once"
    return {"loss": float(loss), "grads": grads, "weights": new_w, "m": new_m, "v": new_v}
