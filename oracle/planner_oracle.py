"""Plain CPU oracle of the paper's host-side planners.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module; only tests/
call it.  It shares no code with the C++ planners of the library and never calls them.

What it computes, in the paper's notation (E experts, D devices grouped into nodes of `dpn`
consecutive devices, a placement P as an E x D 0/1 matrix: P[e][d] = 1 when device d holds the
parameters of expert e):

  * overlap_degree      t = floor(T_attn * bw / Psi)            (Section 4.2, text after Algorithm 1)
  * predict_load        sliding-window mean of the last w load vectors, w = 5 in the paper
                                                                 (Section 4.2, same paragraph)
  * sparse_materialization   Algorithm 1: shard placement P, loads F, overlap degree t, budget m
                             -> materialization plan P' (a superset of P)
  * token_dispatch      Algorithm 3: placement P', token assignment T[e][d] -> plan R[e][d][d']

Each function takes the steps of the paper's listing in its order.  Where the listing names a
sub-step without defining it, the reading taken is (each is a choice of this build):
  * "top t experts by load", "sort by load descending": descending load, equal loads by ascending
    expert id.
  * assignSlotsByLoad(e, totSlots, F): the expert's share of the |D| * m ephemeral slots in
    proportion to its load among the top-t experts, n = floor(totSlots * F[e] / sum of the top-t
    loads), at least 1 while the loads are not all zero, at most the number of devices that do not
    hold e yet (a device holds at most one replica of an expert); 0 when all top-t loads are zero.
  * "distribute n replicas ... prioritizing nodes that do not already hold a replica of e, then
    devices by available slots": one replica at a time, to the device that minimises
    (its node already holds e, -free slots of the device, device id) among the devices that have
    a free slot and do not hold e; stops early when no such device is left.
  * "evenly dispatch x tokens to a set S": floor(x / |S|) to every device of S and one more to
    the first x mod |S| devices of S in ascending device id.
  * the calibration stage and the cost/benefit test around it are not modelled.
"""
from __future__ import annotations

import math
from typing import List, Sequence


def overlap_degree(t_attn: float, bw: float, psi: float) -> int:
    """Expert chunks one link absorbs within the attention window: floor(T_attn * bw / Psi)."""
    if t_attn < 0 or bw < 0 or psi <= 0:
        raise ValueError("need T_attn >= 0, bw >= 0, Psi > 0")
    return int(math.floor(t_attn * bw / psi))


def predict_load(history: Sequence[Sequence[float]], w: int = 5) -> List[float]:
    """Mean of the last min(w, len(history)) load vectors (oldest first in `history`)."""
    if w < 1 or len(history) == 0:
        raise ValueError("need w >= 1 and at least one recorded iteration")
    last = history[-w:]
    E = len(last[0])
    return [sum(float(row[e]) for row in last) / len(last) for e in range(E)]


def _node(d: int, dpn: int) -> int:
    return d // dpn


def sparse_materialization(P: Sequence[Sequence[int]], F: Sequence[float], t: int, m: int, dpn: int):
    """Algorithm 1.  P [E][D] 0/1, F [E] loads, t overlap degree, m ephemeral replicas per device.
    Returns P' [E][D] as lists of 0/1."""
    E, D = len(P), len(P[0])
    if D % dpn != 0 or t < 0 or m < 0 or any(f < 0 for f in F):
        raise ValueError("bad arguments")
    t = min(t, E)
    m = min(m, t)
    Pp = [[1 if P[e][d] else 0 for d in range(D)] for e in range(E)]
    by_load = sorted(range(E), key=lambda e: (-float(F[e]), e))
    top = by_load[:t]                       # already in descending load
    if t <= m:
        for e in top:
            for d in range(D):
                Pp[e][d] = 1
        return Pp
    tot_slots = D * m
    free = [m] * D
    top_load = sum(float(F[e]) for e in top)
    for e in top:
        holders = sum(Pp[e])
        if top_load > 0:
            n = int(math.floor(tot_slots * float(F[e]) / top_load))
            n = max(n, 1)
        else:
            n = 0
        n = min(n, D - holders)
        for _ in range(n):
            cand = [d for d in range(D) if free[d] > 0 and not Pp[e][d]]
            if not cand:
                break
            node_has = {_node(d, dpn) for d in range(D) if Pp[e][d]}
            d = min(cand, key=lambda d: (1 if _node(d, dpn) in node_has else 0, -free[d], d))
            Pp[e][d] = 1
            free[d] -= 1
    return Pp


def token_dispatch(Pp: Sequence[Sequence[int]], T: Sequence[Sequence[int]], dpn: int):
    """Algorithm 3.  P' [E][D] 0/1, T [E][D] tokens of device d assigned to expert e.
    Returns R [E][D][D]: R[e][d][d2] tokens of device d sent to expert e on device d2."""
    E, D = len(Pp), len(Pp[0])
    if D % dpn != 0:
        raise ValueError("devices do not fill whole nodes")
    R = [[[0] * D for _ in range(D)] for _ in range(E)]

    def evenly(x, S):
        q, r = divmod(x, len(S))
        return {d2: q + (1 if i < r else 0) for i, d2 in enumerate(sorted(S))}

    for e in range(E):
        De = [d for d in range(D) if Pp[e][d]]
        if not De:
            raise ValueError(f"expert {e} is materialized nowhere")
        for d in De:                                    # local dispatching
            R[e][d][d] = int(T[e][d])
        for d in range(D):
            if Pp[e][d]:
                continue
            local = [d2 for d2 in range(D) if _node(d2, dpn) == _node(d, dpn)]
            elocal = [d2 for d2 in De if d2 in local]
            target = elocal if elocal else De           # intra-node, else inter-node dispatching
            for d2, x in evenly(int(T[e][d]), target).items():
                R[e][d][d2] = x
    return R
