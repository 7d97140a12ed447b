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
    to the per-pack test (a runtime whose memory need is not a sum over the
    layers of one pack, e.g. because the largest slot and the largest
    activation workspace can come from different packs, passes its own test).
Times and memories are integers.  This module knows nothing of the library's
memory model: the tests hand it the library's own per-layer lists.

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
