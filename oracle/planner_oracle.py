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

Algorithm 1 and Algorithm 3 are heuristics, so the oracle follows what each of them decides, in
the paper's order of decisions (candidates by load, then replica counts, then placement; for the
dispatch: own device, else own node, else everywhere), written as array operations over whole
experts rather than as the listings' statements.  The listings leave some sub-steps to the reader;
the readings taken are choices of this build:
  * ranking experts by load: descending load, equal loads by ascending expert id.
  * the number of new replicas of a candidate (the listing only names a helper for it): its share of
    the |D| * m ephemeral slots in proportion to its load among the t candidates, rounded down, at
    least 1 while those loads are not all zero, never more than the devices that lack the expert
    (a device holds an expert at most once); 0 when all candidate loads are zero.
  * where the new replicas go (the listing states two priorities and no procedure): one at a time,
    to a device that lacks the expert and has a free slot, preferring first a node where the expert
    is absent, then the device with the most free slots, then the lowest device id; placement of
    an expert stops when no such device is left.
  * an even split of x tokens over n devices: x // n each, and one more for the x mod n lowest
    device ids.
  * the calibration stage and the cost/benefit test around it are not modelled.
"""
from __future__ import annotations

import math
from typing import Dict, List, Sequence

import numpy as np


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


def replica_counts(P: np.ndarray, F: np.ndarray, cand: Sequence[int], slots: int) -> Dict[int, int]:
    """New replicas each candidate of Algorithm 1 is entitled to: proportional to load, see the header."""
    D = P.shape[1]
    load = float(sum(F[e] for e in cand))
    out = {}
    for e in cand:
        share = max(1, int(math.floor(slots * float(F[e]) / load))) if load > 0 else 0
        out[e] = min(share, D - int(P[e].sum()))
    return out


def sparse_materialization(P: Sequence[Sequence[int]], F: Sequence[float], t: int, m: int, dpn: int):
    """Algorithm 1 (Sparse Materialization).  P [E][D] 0/1 shard placement, F [E] loads, t overlap
    degree, m ephemeral replicas per device.  Returns the plan P' [E][D] as lists of 0/1."""
    plan = (np.asarray(P) != 0).astype(np.int64)
    E, D = plan.shape
    load = np.asarray(F, dtype=np.float64)
    if D % dpn != 0 or t < 0 or m < 0 or (load < 0).any():
        raise ValueError("bad arguments")
    t = min(t, E)
    m = min(m, t)
    # candidates: the t most loaded experts (a stable sort on the negated load keeps equal loads in id order)
    cand = [int(e) for e in np.argsort(-load, kind="stable")[:t]]
    if t <= m:
        plan[cand, :] = 1            # room for every candidate on every device
        return plan.tolist()
    want = replica_counts(plan, load, cand, D * m)
    free = np.full(D, m, dtype=np.int64)
    node_of = np.arange(D) // dpn
    for e in cand:                   # heaviest first: it chooses among the most free slots
        for _ in range(want[e]):
            open_dev = np.flatnonzero((free > 0) & (plan[e] == 0))
            if open_dev.size == 0:
                break
            node_has_e = np.isin(node_of[open_dev], node_of[plan[e] == 1])
            # lexicographic preference: absent from the node, most free slots, lowest id
            order = np.lexsort((open_dev, -free[open_dev], node_has_e))
            d = int(open_dev[order[0]])
            plan[e, d] = 1
            free[d] -= 1
    return plan.tolist()


def split_evenly(x: int, n: int) -> List[int]:
    """x tokens over n receivers in ascending id: x // n each, the first x mod n get one more."""
    return [x // n + (1 if i < x % n else 0) for i in range(n)]


def token_dispatch(Pp: Sequence[Sequence[int]], T: Sequence[Sequence[int]], dpn: int):
    """Algorithm 3 (Topology-aware Token Dispatching).  P' [E][D] 0/1, T [E][D] tokens of device d
    assigned to expert e.  Returns R [E][D][D]: R[e][d][d2] tokens of device d sent to expert e on d2."""
    held = np.asarray(Pp) != 0
    tokens = np.asarray(T, dtype=np.int64)
    E, D = held.shape
    if D % dpn != 0:
        raise ValueError("devices do not fill whole nodes")
    node_of = np.arange(D) // dpn
    R = np.zeros((E, D, D), dtype=np.int64)
    for e in range(E):
        if not held[e].any():
            raise ValueError(f"expert {e} is materialized nowhere")
        for d in range(D):
            # receivers of device d's tokens for e, by decreasing locality: itself, the holders in its
            # node, all holders -- the first of the three sets that is not empty
            for level in (held[e] & (np.arange(D) == d), held[e] & (node_of == node_of[d]), held[e]):
                recv = np.flatnonzero(level)
                if recv.size:
                    break
            R[e, d, recv] = split_evenly(int(tokens[e, d]), recv.size)
    return R.tolist()
