"""Event-driven simulation of one iteration's task list (the paper's Runtime
Estimator, Section 4.3.1: "an event-driven simulation to capture swap, transfer
and compute times" over the task graph, fed with per-layer profiles).

TEST INFRASTRUCTURE.  Two parts, neither of which knows the library:

  run(ops)            a generic simulator of FIFO resources.  An operation names its
                      resource, its duration and what it waits for; each resource
                      serves its operations one at a time in the order they are listed.
  iteration_ops(...)  turns the ordered task list of `schedule.task_list` (Algorithm 3
                      at N = 1) into such operations on the resources of Section 4.4:
                      the compute stream, the swap-in stream (host -> device link), the
                      swap-out stream (device -> host link) and, when the Weight Update
                      runs there, the CPU.

The paper gives the estimator's role and inputs, not its rules; the rules below are
this build's reading of Section 4.4 (prefetch, double buffering, jit-update) at task
granularity.  A "visit" is a forward or backward task; visit v owns weight slot
v mod S of S slots.

  compute   C(v): on the compute stream, n_microbatches x (sum of the pack's per-layer
            times); needs the weights W(v).
  weights   W(v): on the swap-in stream, w_c bytes per parameter.  Prefetch distance D:
            W(v + D) is requested when C(v) starts (W(0..D-1) at time 0), and it needs
            its slot: the visit S places earlier must have left it -- a forward visit
            when its compute ends, a backward visit when its update has been written
            back.  A request that waits holds up the requests queued behind it.
  stash     a forward visit sends one checkpoint per microbatch for every backward-pack
            input among its layers (swap-out stream); a backward visit that restarts
            from a checkpoint reads one per microbatch (swap-in stream).  They travel
            while their visit computes: requested when C(v) starts.  Nothing waits for the
            ones going out; the ones coming in are the visit's input (Section 4.3.1: the
            backward task recomputes from the stashed pack input), so C(v) cannot end
            before they have all arrived -- behind whatever the swap-in stream was asked
            for earlier, such as the optimizer state of the update before.
  update    after C(v) of a backward visit (jit-update).  On the device: the optimizer
            state K(v) comes in (k_B bytes per parameter, swap-in stream, requested when
            C(v) ends, behind whatever was requested earlier); state, weights and the
            exported gradient go out as one operation (swap-out stream) that starts when
            C(v) ends and cannot end before K(v) has arrived.  On the host: only the
            gradient goes out, then the CPU applies the update (its own queue).
  result    the time the last operation ends.
  slowdown  (optional) kernels run slower while the device->host link is busy beside them.  Given
            a second set of per-layer times taken beside link traffic, a visit's compute time is
            its time alone plus the difference to that second time, in proportion to the share of
            its time alone for which the device->host link still has work queued when it starts
            (what earlier updates left unfinished, plus its own checkpoints), at most all of it.

Pins (tests/test_oracle_schedule.py): schedules worked by hand; with a link of
unbounded speed the result is the sum of the compute times, with unbounded compute
it is the busier link's serial time; more slots or a faster link never lengthen it.
Parity unpinned: agreement with measured iteration times (that is a property of the
hardware, reported in the benchmark's notes, not something the CPU tests can fix).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from fractions import Fraction

from . import model as om
from . import schedule as osch


@dataclass
class Op:
    """One operation.  after_end: operations that must have ended before it starts;
    after_start: operations that must have started; not_before_end: operations it
    cannot end before (it runs at their pace if they are slower)."""
    name: str
    resource: str
    duration: Fraction
    after_end: list = field(default_factory=list)
    after_start: list = field(default_factory=list)
    not_before_end: list = field(default_factory=list)
    # (resource, duration beside a busy resource): the operation takes `duration` if that resource is idle
    # when it starts and stretches towards the second figure in proportion to the share of `duration` for
    # which the operations listed before it on that resource still keep it busy
    stretch: tuple | None = None


def run(ops):
    """Start and end time of every operation: {name: (start, end)}.  Each resource
    serves its operations in list order, one at a time."""
    by_name = {o.name: o for o in ops}
    assert len(by_name) == len(ops), "operation names must be unique"
    prev_on_resource = {}
    last_listed = {}          # per operation: the last operation listed before it on each resource
    last = {}
    for o in ops:
        prev_on_resource[o.name] = last.get(o.resource)
        last_listed[o.name] = dict(last)
        last[o.resource] = o.name
    starts, times = {}, {}
    visiting = set()

    def start_of(name):
        if name in starts:
            return starts[name]
        assert name not in visiting, f"dependency cycle through {name}"
        visiting.add(name)
        o = by_name[name]
        start = Fraction(0)
        if prev_on_resource[name] is not None:
            start = max(start, solve(prev_on_resource[name])[1])
        for d in o.after_end:
            start = max(start, solve(d)[1])
        for d in o.after_start:
            start = max(start, start_of(d))
        visiting.discard(name)
        starts[name] = start
        return start

    def solve(name):
        if name in times:
            return times[name]
        o = by_name[name]
        start = start_of(name)
        duration = o.duration
        if o.stretch is not None and o.duration > 0:
            resource, beside = o.stretch
            before = last_listed[name].get(resource)
            backlog = max(Fraction(0), solve(before)[1] - start) if before is not None else Fraction(0)
            duration = o.duration + (Fraction(beside) - o.duration) * min(Fraction(1), backlog / o.duration)
        end = start + duration
        for d in o.not_before_end:
            end = max(end, solve(d)[1])
        times[name] = (start, end)
        return times[name]

    import sys
    old = sys.getrecursionlimit()
    sys.setrecursionlimit(max(old, 10 * len(ops) + 1000))
    try:
        for o in ops:
            solve(o.name)
    finally:
        sys.setrecursionlimit(old)
    return times


def iteration_ops(spec: om.Spec, P_F, P_B, t_fwd, t_bwd, M_F: int, M_B: int, act_bytes_F: int, act_bytes_B: int,
                  w_c: int, k_B: int, g_B: int, ns_per_byte_in, ns_per_byte_out, slots: int = 3, distance: int = 1,
                  update_on_host: bool = False, host_ns_per_param=Fraction(1, 6), export_gradients: bool = True,
                  t_fwd_beside=None, t_bwd_beside=None):
    """Operations of one layer-pack-major iteration.

    t_fwd[l], t_bwd[l]: time of layer l for ONE microbatch of the forward / backward
    microbatch size (t_bwd = recompute + backward, or forward + backward for the last
    pack); M_F, M_B: microbatches per pass; act_bytes_F / act_bytes_B: bytes of one
    microbatch's checkpoint in each pass.  t_fwd_beside / t_bwd_beside: the same times
    taken beside link traffic (the slowdown rule); None = no slowdown."""
    assert slots >= 2 and 1 <= distance < slots
    tasks = osch.task_list(spec, P_F, P_B)
    visits = [t for t in tasks if t.kind in "FB"]
    npar = lambda t: sum(om.layer_param_count(spec, l) for l in range(*t.pack))
    F = Fraction
    ops = []
    left_slot = {}            # visit index -> name of the operation after which its slot is free

    def weights(v):
        deps = []
        if v - slots >= 0:
            deps.append(left_slot[v - slots])
        gate = [f"C{v - distance}"] if v - distance >= 0 else []
        ops.append(Op(f"W{v}", "h2d", F(w_c * npar(visits[v])) * ns_per_byte_in, after_end=deps, after_start=gate))

    # Operations are listed in the order the runtime would request them, which is the
    # order each stream serves them in.  W(v + D) is requested when C(v) starts, K(v)
    # when C(v) ends, so K(v) is listed behind W(v + D); left_slot of the visit S places
    # before v + D is known by then because D < S.
    for v in range(min(distance, len(visits))):
        weights(v)
    for v, t in enumerate(visits):
        P = npar(t)
        if t.kind == "F":
            dur = M_F * sum(F(t_fwd[l]) for l in range(*t.pack))
            beside = M_F * sum(F(t_fwd_beside[l]) for l in range(*t.pack)) if t_fwd_beside is not None else None
        else:
            dur = M_B * sum(F(t_bwd[l]) for l in range(*t.pack))
            beside = M_B * sum(F(t_bwd_beside[l]) for l in range(*t.pack)) if t_bwd_beside is not None else None
        if t.kind == "B" and t.stash_in_layer is not None:
            ops.append(Op(f"Sin{v}", "h2d", F(M_B * act_bytes_B) * ns_per_byte_in, after_start=[f"C{v}"]))
        if t.kind == "F" and t.stash_out_layers:
            ops.append(Op(f"Sout{v}", "d2h", F(len(t.stash_out_layers) * M_F * act_bytes_F) * ns_per_byte_out,
                          after_start=[f"C{v}"]))
        ops.append(Op(f"C{v}", "comp", dur, after_end=[f"W{v}"],
                      not_before_end=[f"Sin{v}"] if t.kind == "B" and t.stash_in_layer is not None else [],
                      stretch=("d2h", beside) if beside is not None else None))
        if t.kind == "F":
            left_slot[v] = f"C{v}"
        elif update_on_host:
            ops.append(Op(f"Out{v}", "d2h", F(g_B * P) * ns_per_byte_out, after_end=[f"C{v}"]))
            ops.append(Op(f"Cpu{v}", "cpu", F(P) * host_ns_per_param, after_end=[f"Out{v}"]))
            left_slot[v] = f"Out{v}"
        else:
            out_bytes = (k_B + w_c + (g_B if export_gradients else 0)) * P
            ops.append(Op(f"Out{v}", "d2h", F(out_bytes) * ns_per_byte_out, after_end=[f"C{v}"],
                          not_before_end=[f"K{v}"]))
            left_slot[v] = f"Out{v}"
        if v + distance < len(visits):
            weights(v + distance)
        if t.kind == "B" and not update_on_host:
            ops.append(Op(f"K{v}", "h2d", F(k_B * P) * ns_per_byte_in, after_end=[f"C{v}"]))
    return ops


def iteration_time(*args, **kwargs):
    """End of the last operation of iteration_ops(...)."""
    times = run(iteration_ops(*args, **kwargs))
    return max(e for (_, e) in times.values())
