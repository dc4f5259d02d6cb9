"""Pins of the planner oracle (oracle/planner_oracle.py): hand-worked cases, closed forms, invariants
that follow from the text of Algorithms 1 and 3, and planted mistakes.  CPU only.

The paper prints no worked numeric example of either algorithm; the hand-worked cases below are
derived from the listings with the readings stated in the oracle's header.
"""
from __future__ import annotations

import numpy as np
import pytest

from oracle import planner_oracle as po


def _ident(E, D):
    return [[1 if d == e % D else 0 for d in range(D)] for e in range(E)]


def _check_dispatch_rules(Pp, T, R, dpn):
    """The properties Algorithm 3's text states, checked without recomputing the plan."""
    E, D = len(Pp), len(Pp[0])
    for e in range(E):
        holders = [d for d in range(D) if Pp[e][d]]
        for d in range(D):
            row = R[e][d]
            assert sum(row) == T[e][d]                               # every token goes somewhere
            assert all(x >= 0 for x in row)
            assert all(x == 0 for d2, x in enumerate(row) if not Pp[e][d2])   # only to holders
            if Pp[e][d]:
                assert row[d] == T[e][d]                             # local dispatching
                continue
            same_node = [d2 for d2 in holders if d2 // dpn == d // dpn]
            target = same_node if same_node else holders
            assert all(x == 0 for d2, x in enumerate(row) if d2 not in target)  # intra-node when possible
            got = [row[d2] for d2 in target]
            assert max(got) - min(got) <= 1                          # evenly
            assert got == sorted(got, reverse=True)                  # the extra tokens to the lowest ids


def _pins():
    # ---- overlap degree: 2 ms window, 50 GB/s, 88 MB per expert -> floor(1.135..) = 1; exact multiples
    assert po.overlap_degree(2e-3, 50e9, 88_080_384) == 1
    assert po.overlap_degree(1.0, 8.0, 2.0) == 4
    assert po.overlap_degree(1.0, 7.9, 2.0) == 3
    assert po.overlap_degree(0.0, 1e9, 1.0) == 0
    # ---- load prediction: mean of the last 5 (or fewer) iterations
    hist = [[10, 0], [1, 1], [2, 3], [3, 5], [4, 7], [5, 9]]
    assert po.predict_load(hist, 5) == [3.0, 5.0]
    assert po.predict_load(hist[:2], 5) == [5.5, 0.5]
    assert po.predict_load(hist, 1) == [5.0, 9.0]

    # ---- Algorithm 3, hand-worked.  4 devices in nodes {0,1},{2,3}; expert 0 on device 1 only
    R = po.token_dispatch([[0, 1, 0, 0]], [[3, 5, 7, 4]], 2)
    assert R[0] == [[0, 3, 0, 0], [0, 5, 0, 0], [0, 7, 0, 0], [0, 4, 0, 0]]
    # 6 devices in nodes {0,1,2},{3,4,5}; holders 1, 2, 3: device 0 splits 5 over {1, 2} (3 + 2),
    # devices 4 and 5 send everything to 3, holders keep their own
    R = po.token_dispatch([[0, 1, 1, 1, 0, 0]], [[5, 6, 7, 8, 9, 2]], 3)
    assert R[0] == [[0, 3, 2, 0, 0, 0], [0, 6, 0, 0, 0, 0], [0, 0, 7, 0, 0, 0], [0, 0, 0, 8, 0, 0],
                    [0, 0, 0, 9, 0, 0], [0, 0, 0, 2, 0, 0]]
    # no holder in the sender's node: 7 tokens of device 3 over all holders {0, 1}: 4 + 3
    R = po.token_dispatch([[1, 1, 0, 0]], [[1, 1, 0, 7]], 2)
    assert R[0][3] == [4, 3, 0, 0] and R[0][2] == [0, 0, 0, 0]
    with pytest.raises(ValueError):
        po.token_dispatch([[0, 0]], [[1, 1]], 2)
    # ---- Algorithm 3, the rules of its text on random instances
    rng = np.random.default_rng(5)
    for _ in range(40):
        dpn = int(rng.choice([1, 2, 4]))
        D = dpn * int(rng.integers(1, 4))
        E = int(rng.integers(1, 7))
        Pp = (rng.random((E, D)) < 0.35).astype(int)
        for e in range(E):
            Pp[e, rng.integers(0, D)] = 1
        T = rng.integers(0, 50, size=(E, D))
        R = po.token_dispatch(Pp.tolist(), T.tolist(), dpn)
        _check_dispatch_rules(Pp.tolist(), T.tolist(), R, dpn)

    # ---- Algorithm 1, first branch (t <= m): the top-t experts on every device
    P = _ident(4, 4)
    Pp = po.sparse_materialization(P, [5, 1, 9, 3], t=2, m=3, dpn=2)
    assert Pp == [[1, 1, 1, 1], [0, 1, 0, 0], [1, 1, 1, 1], [0, 0, 0, 1]]
    # t larger than the number of experts is clipped: everything everywhere
    assert po.sparse_materialization(P, [1, 1, 1, 1], t=9, m=9, dpn=2) == [[1] * 4] * 4
    # equal loads: the lower expert ids are taken
    assert po.sparse_materialization(P, [2, 2, 2, 2], t=1, m=1, dpn=2)[0] == [1, 1, 1, 1]
    # ---- Algorithm 1, second branch, hand-worked: experts 0..3 on devices 0..3 (nodes {0,1},{2,3}),
    # loads 8, 1, 4, 3, t = 3, m = 1: top = (0, 2, 3), 4 slots; expert 0 gets floor(4*8/15) = 2
    # replicas: first the node without it (device 2), then device 1; expert 2 gets 1: device 0
    # (node without it); expert 3 gets max(floor(4*3/15), 1) = 1 but no device with a free slot
    # that lacks it is left.
    Pp = po.sparse_materialization(P, [8, 1, 4, 3], t=3, m=1, dpn=2)
    assert Pp == [[1, 1, 1, 0], [0, 1, 0, 0], [1, 0, 1, 0], [0, 0, 0, 1]]
    # the same with m = 2 (8 slots): expert 0: floor(8*8/15) = 4 -> capped at the 3 devices that lack it
    Pp = po.sparse_materialization(P, [8, 1, 4, 3], t=3, m=2, dpn=2)
    assert Pp[0] == [1, 1, 1, 1] and Pp[1] == [0, 1, 0, 0]
    assert sum(Pp[2]) == 1 + 2 and sum(Pp[3]) == 1 + 1      # floor(8*4/15) = 2, floor(8*3/15) = 1
    # all loads zero: nothing to balance in the second branch
    assert po.sparse_materialization(P, [0, 0, 0, 0], t=3, m=1, dpn=2) == P
    # ---- Algorithm 1, invariants on random instances
    for _ in range(60):
        dpn = int(rng.choice([1, 2, 4]))
        D = dpn * int(rng.integers(1, 5))
        E = int(rng.integers(1, 12))
        P = _ident(E, D)
        F = rng.integers(0, 100, size=E).astype(float).tolist()
        t, m = int(rng.integers(0, E + 3)), int(rng.integers(0, 5))
        Pp = po.sparse_materialization(P, F, t, m, dpn)
        te, me = min(t, E), min(m, min(t, E))
        order = sorted(range(E), key=lambda e: (-F[e], e))
        top = set(order[:te])
        added = [[Pp[e][d] - P[e][d] for d in range(D)] for e in range(E)]
        assert all(a in (0, 1) for row in added for a in row)         # P' is a superset of P
        assert all(sum(added[e]) == 0 for e in range(E) if e not in top)   # only the top-t gain replicas
        if te <= me:
            assert all(sum(Pp[e]) == D for e in top)
        else:
            assert all(sum(added[e][d] for e in range(E)) <= me for d in range(D))   # budget per device
            tl = sum(F[e] for e in top)
            for e in top:
                want = min(D - sum(P[e]), max(1, int(me * D * F[e] // tl))) if tl > 0 else 0
                assert sum(added[e]) <= want                            # never more than its share
            # the most loaded expert is placed first, with every slot still free: each new replica
            # goes to a node that lacks the expert until every node has one
            first = order[0]
            gained = sum(added[first])
            nodes_with = {d // dpn for d in range(D) if Pp[first][d]}
            assert len(nodes_with) == min(D // dpn, 1 + gained)


def test_planner_pins():
    _pins()


def test_planted_mistakes_in_planners_are_caught(monkeypatch):
    real_sm, real_td = po.sparse_materialization, po.token_dispatch

    def td_always_all_holders(Pp, T, dpn):            # intra-node branch dropped: one node of all devices
        return real_td(Pp, T, len(Pp[0]))

    def td_remainder_to_last(Pp, T, dpn):             # the extra tokens to the highest device ids
        R = real_td(Pp, T, dpn)
        for e in range(len(Pp)):
            for d in range(len(Pp[0])):
                if not Pp[e][d]:
                    targets = [d2 for d2, x in enumerate(R[e][d]) if x > 0]
                    for d2, v in zip(targets, [R[e][d][q] for q in reversed(targets)]):
                        R[e][d][d2] = v
        return R

    def sm_ties_to_higher_id(P, F, t, m, dpn):        # equal loads broken towards the higher expert id
        return real_sm(P[::-1], list(F)[::-1], t, m, dpn)[::-1]

    def sm_bigger_share(P, F, t, m, dpn):             # a slot more per device than the budget allows
        return real_sm(P, F, t, m + 1, dpn) if min(t, len(P)) > m else real_sm(P, F, t, m, dpn)

    def sm_no_topology(P, F, t, m, dpn):              # node priority dropped: one node of all devices
        return real_sm(P, F, t, m, len(P[0]))

    for name, bad in (("token_dispatch", td_always_all_holders), ("token_dispatch", td_remainder_to_last),
                      ("sparse_materialization", sm_ties_to_higher_id), ("sparse_materialization", sm_bigger_share),
                      ("sparse_materialization", sm_no_topology)):
        with monkeypatch.context() as mp:
            mp.setattr(po, name, bad)
            with pytest.raises((AssertionError, ValueError)):
                _pins()
    _pins()
